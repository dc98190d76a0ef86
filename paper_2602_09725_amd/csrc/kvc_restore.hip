// Restore kernels: unpack frames, dequantize, place (Sec. 3.3.2 "Frame-wise KV
// tensor restoration"; Sec. 4 item (2), the frame-to-paged-memory transfer).
//
// One fused kernel does all three steps in a single pass over the data, so the
// HBM traffic is the algorithmic minimum: 1 byte of code read and 2 bytes of
// fp16/bf16 written per element, plus the scale/min pairs.  The path is purely
// bandwidth bound; there is no contraction in it, hence no MFMA.
//
// Work decomposition.  An "atom" is 8 consecutive elements of a token's H*D
// vector: 8 code bytes in one frame row (tile_w % 8 == 0) that belong to one
// head (head_dim % 8 == 0), restored to 16 contiguous bytes.  A workgroup owns a
// contiguous block of tokens of one (chunk, kind, layer); a thread keeps one atom
// for the whole block, so
//   - a wave's store covers 1024 contiguous output bytes and its load whole
//     128-byte (or longer) runs of a frame row: full cache lines both ways,
//   - per-channel scale/min of the thread's 8 channels are loaded once and stay
//     in 16 VGPRs.
// A contiguous block of tokens touches F frames at TX-adjacent tile positions,
// i.e. a few contiguous runs of th rows in each of F planes (Sec. 3.2.1 step 3).
//
// Three bodies:
//  * "rows" (chunk calls on tiles narrower than 512 bytes, e.g. the (8,128) tile of the paper's GQA shapes): a
//    wave reads runs of 512 bytes along a plane row -- the same row of 512 / tw neighbouring tiles, which hold
//    tokens F positions apart (Sec. 3.2.1 step 3) -- and writes tw * 2 bytes of each of those tokens; the th waves
//    of a workgroup take the th rows of the tiles, so together they write whole tokens.  Reads as long as this
//    are what a kernel needs to draw the full rate from pinned host memory over PCIe (128-byte pieces reach 80 % of
//    it), and they suit HBM at least as well as the "waves" body's.
//  * "waves" (C/8 a multiple of 64, every model shape of the paper): a wave works
//    on one token at a time, so everything that depends on the token only (frame,
//    tile position, cache slot, block-table entry, pair address) is the same for
//    all its lanes.  Lane k of the wave computes those values for the wave's k-th
//    token, all tokens at once, and the loop over tokens fetches them with
//    v_readlane.  The per-token cost is then a handful of instructions; with the
//    index arithmetic in the loop the kernel is bound by instruction issue, not by
//    HBM.
//  * "lanes" (any other C): every lane does its own index arithmetic.
#include <hip/hip_runtime.h>

#include "kvc_device.h"
#include "kvc_launch.h"

namespace kvc {

#ifndef KVC_RESTORE_U
#define KVC_RESTORE_U 8  // tokens in flight per wave
#endif
#ifndef KVC_RESTORE_TB
#define KVC_RESTORE_TB 32  // tokens per workgroup ("waves" body)
#endif
#ifndef KVC_RESTORE_TB_LANES
#define KVC_RESTORE_TB_LANES 128  // tokens per workgroup ("lanes" body)
#endif

namespace {

__device__ __forceinline__ uint32_t lane_value(uint32_t v, uint32_t k) {
  return (uint32_t)__builtin_amdgcn_readlane((int)v, (int)k);
}

// 8 codes -> 8 dequantized 16-bit values, one 16-byte store.
template <int MODE, int DT>
__device__ __forceinline__ void dequant_store(uint16_t* dst, u32x2 code, const float (&sc)[8], const float (&mn)[8],
                                              f32x2 sm) {
  float x[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t w = i < 4 ? code.x : code.y;
    const float q = (float)((w >> (8 * (i & 3))) & 0xffu);
    x[i] = MODE == KVC_Q_PER_CHANNEL ? __builtin_fmaf(q, sc[i], mn[i]) : __builtin_fmaf(q, sm.x, sm.y);
    // The dequantized value is defined as the binary32 fma result, then rounded
    // to 16 bits.  Keep the two roundings apart: a mixed-precision fma that
    // rounds the exact sum straight to fp16 differs in about 1 value in 10^4.
    asm("" : "+v"(x[i]));
  }
  u32x4 o;
  o.x = narrow_pair<DT>(x[0], x[1]);
  o.y = narrow_pair<DT>(x[2], x[3]);
  o.z = narrow_pair<DT>(x[4], x[5]);
  o.w = narrow_pair<DT>(x[6], x[7]);
  stream_store<u32x4>(dst, o);
}

// Scale/min of the 8 channels of atom e (per-channel grouping).
__device__ __forceinline__ void load_channel_pairs(const float* mbase, int64_t first_pair, float (&sc)[8], float (&mn)[8]) {
  const KVC_GLOBAL f32x2* mp = (const KVC_GLOBAL f32x2*)(mbase + 2 * first_pair);
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const f32x2 v = mp[i];
    sc[i] = v.x;
    mn[i] = v.y;
  }
}

// ----------------------------------------------------------------- "waves" body

template <int MODE, int DT, bool PAGED>
__device__ __forceinline__ void restore_body_waves(const RestoreParams& p, uint32_t c, uint32_t kind, uint32_t l,
                                                   uint32_t tbi, const uint8_t* fsec, uint32_t ff) {
  constexpr int U = KVC_RESTORE_U;
  const Geo& g = p.g;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t wave = wave_uniform(threadIdx.x >> 6);
  const uint32_t tsub = fd_div(p.dwpt, wave);              // which token of a pass this wave takes
  const uint32_t wslab = wave - tsub * p.dwpt.d;           // which 64-atom part of the token
  const uint32_t e = (wslab * 64u + lane) * 8u;            // first element of the lane's atom

  const int64_t chunk_first = (int64_t)c * g.T;
  const int64_t left = p.n_tokens - chunk_first;
  const int32_t n = left < (int64_t)g.T ? (int32_t)left : g.T;  // valid tokens of this chunk
  // Token slots of this workgroup: tb consecutive slots; pass k of this wave takes slot
  // t0 + tsub + k * tpp.  Slot s is token s (chunk call) or token s * F + f (frame call:
  // only the tokens whose tile sits in frame f of their group, Sec. 3.2.1 step 3).
  const int32_t ns = p.frame_mode ? (n > (int32_t)ff ? (n - (int32_t)ff + g.F - 1) / g.F : 0) : n;
  const int32_t t0 = (int32_t)tbi * p.tb;
  const int32_t t1 = t0 + p.tb < ns ? t0 + p.tb : ns;
  if (t0 >= t1) return;
  const int32_t t = t0 + (int32_t)tsub + (int32_t)lane * p.tpp;
  const bool in_range = t < t1;
  const uint32_t tslot = (uint32_t)(in_range ? t : t0);  // clamp: loads of dead passes stay in bounds
  const uint32_t tc = p.frame_mode ? tslot * (uint32_t)g.F + ff : tslot;
  // inter-frame layout: token -> (frame of its group, tile position of its group)
  uint32_t gi, f, ty, tx;
  fd_divmod(g.dF, tc, gi, f);
  fd_divmod(g.dTX, gi, ty, tx);
  const uint32_t src_tok = f * p.frame_stride + ty * p.tile_row_stride + tx * (uint32_t)g.tw;  // bytes inside the section
  uint64_t dst_tok;  // bytes from the layer's (kind) base
  bool ok = in_range;
  if (PAGED) {
    uint32_t b, slot;
    fd_divmod(p.dbs, (uint32_t)(p.first_token + chunk_first) + tc, b, slot);
    const int32_t phys = as_const(p.table)[b];
    const bool in_cache = (uint32_t)phys < (uint32_t)p.num_blocks;
    // an id outside the cache: skip the block's writes and report it (Sec. 3.3.2 placement)
    if (in_range && !in_cache && wslab == 0 && p.err) atomicOr(p.err, 1u);
    ok = in_range && in_cache;
    dst_tok = ((uint64_t)(in_cache ? (uint32_t)phys : 0u) * p.dbs.d + slot) * (uint32_t)g.C * 2u;
  } else {
    dst_tok = (uint64_t)tc * (uint64_t)p.ts * 2u;
  }
  const uint64_t live_mask = __ballot(ok);
  const uint32_t passes = (uint32_t)__popcll(__ballot(in_range));  // in_range is a prefix of the lanes
  const uint32_t dst_lo = (uint32_t)dst_tok, dst_hi = (uint32_t)(dst_tok >> 32);

  // ---- per-lane constants
  uint32_t r, cc;
  tile_pos(g, e, r, cc);  // intra-frame layout: element -> (row, column) of the tile
  const uint32_t src_lane = r * (uint32_t)g.W + cc;
  const float* mbase = p.meta + (int64_t)c * g.meta_floats + p.moff[kind];
  const uint32_t lm = l - (uint32_t)p.meta_l0;  // layer index inside the pairs that `meta` holds
  float sc[8], mn[8];
  const uint8_t* mrow = nullptr;
  if (MODE == KVC_Q_PER_CHANNEL) {
    load_channel_pairs(mbase, (int64_t)lm * g.C + e, sc, mn);
  } else {
    mrow = reinterpret_cast<const uint8_t*>(mbase + 2 * ((int64_t)lm * g.T * g.H + fd_div(g.dD, e)));
  }
  uint8_t* obase;
  if (PAGED)
    obase = reinterpret_cast<uint8_t*>(as_const(p.layer_cache)[l]) + ((int64_t)kind * p.num_blocks * p.dbs.d * g.C + e) * 2;
  else
    obase = reinterpret_cast<uint8_t*>(p.out + (int64_t)l * p.ls + (int64_t)kind * p.ks + chunk_first * p.ts + e);

  // ---- the tokens of this wave, U at a time
  for (uint32_t k0 = 0; k0 < passes; k0 += U) {
    u32x2 code[U];
    f32x2 sm[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t k = k0 + u < passes ? k0 + u : passes - 1;
      code[u] = stream_load<u32x2>(fsec + (lane_value(src_tok, k) + src_lane));
      if (MODE == KVC_Q_PER_TOKEN)
        sm[u] = *(const KVC_GLOBAL f32x2*)(mrow + (size_t)lane_value(tc, k) * ((uint32_t)g.H * 8u));
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t k = k0 + u;
      if (k >= passes || !((live_mask >> k) & 1ull)) continue;  // wave-uniform
      const uint64_t off = ((uint64_t)lane_value(dst_hi, k) << 32) | lane_value(dst_lo, k);
      dequant_store<MODE, DT>(reinterpret_cast<uint16_t*>(obase + off), code[u], sc, mn, sm[u]);
    }
  }
}

// ------------------------------------------------------------------ "rows" body

// First element of the atom at (row r, column cc) of a token's tile: the inverse of tile_pos.
__device__ __forceinline__ uint32_t tile_elem(const Geo& g, uint32_t r, uint32_t cc) {
  if (g.seg == 0) return r * (uint32_t)g.tw + cc;
  const uint32_t a = r / (uint32_t)g.d1, c = r - a * (uint32_t)g.d1;
  const uint32_t b = fd_div(g.dseg, cc), i = cc - b * (uint32_t)g.seg;
  return (a * g.dh2.d + b) * (uint32_t)g.D + c * (uint32_t)g.seg + i;
}

// Unit `tg` is a group of rows_trw rows of tiles of one (chunk, kind, layer), in all F frames (chunk call) or in
// frame ff alone (frame call: fsec is then that frame's plane and frame_stride 0).
template <int MODE, int DT, bool PAGED>
__device__ __forceinline__ void restore_body_rows(const RestoreParams& p, uint32_t c, uint32_t kind, uint32_t l,
                                                  uint32_t tg, const uint8_t* fsec, uint32_t ff) {
  constexpr int U = KVC_RESTORE_U;
  const Geo& g = p.g;
  const uint32_t lane = threadIdx.x & 63u;
  const uint32_t r = wave_uniform(threadIdx.x >> 6);       // row of the tiles this wave reads
  const uint32_t tl = lane >> (uint32_t)p.rows_lat;         // which of the q tiles of a run the lane is in
  const uint32_t cc = (lane - (tl << (uint32_t)p.rows_lat)) * 8u;
  const uint32_t e = tile_elem(g, r, cc);

  const int64_t chunk_first = (int64_t)c * g.T;
  const int64_t left = p.n_tokens - chunk_first;
  const uint32_t n = left < (int64_t)g.T ? (uint32_t)left : (uint32_t)g.T;  // valid tokens of this chunk
  const uint32_t per_row = (uint32_t)g.TX * (uint32_t)g.F;                   // tokens of one row of tiles
  const uint32_t ty0 = tg * (uint32_t)p.rows_trw;                            // first row of tiles of this unit
  if (ty0 >= (uint32_t)p.rows_tile_rows || ty0 * per_row + ff >= n) return;

  const float* mbase = p.meta + (int64_t)c * g.meta_floats + p.moff[kind];
  const uint32_t lm = l - (uint32_t)p.meta_l0;
  float sc[8], mn[8];
  const uint8_t* mrow = nullptr;
  if (MODE == KVC_Q_PER_CHANNEL) {
    load_channel_pairs(mbase, (int64_t)lm * g.C + e, sc, mn);
  } else {
    mrow = reinterpret_cast<const uint8_t*>(mbase + 2 * ((int64_t)lm * g.T * g.H + fd_div(g.dD, e)));
  }
  uint8_t* obase;
  if (PAGED)
    obase = reinterpret_cast<uint8_t*>(as_const(p.layer_cache)[l]) + ((int64_t)kind * p.num_blocks * p.dbs.d * g.C + e) * 2;
  else
    obase = reinterpret_cast<uint8_t*>(p.out + (int64_t)l * p.ls + (int64_t)kind * p.ks + chunk_first * p.ts + e);
  const uint8_t* src = fsec + ((ty0 * (uint32_t)g.th + r) * (uint32_t)g.W + lane * 8u);
  const uint32_t tile0 = ty0 * (uint32_t)g.TX + tl;  // the lane's tile in run 0 of the unit's first row
  const uint32_t pos0 = (uint32_t)(p.first_token + chunk_first);
  // pass k: frame k % nf, run (k / nf) % runs of row of tiles k / (nf * runs); nf = F, or 1 in a frame call
  const uint32_t rows_left = (uint32_t)p.rows_tile_rows - ty0;
  const uint32_t passes = (rows_left < (uint32_t)p.rows_trw ? rows_left : (uint32_t)p.rows_trw) * p.dpr.d;
  const uint32_t row_bytes = (uint32_t)g.th * (uint32_t)g.W;
  bool bad = false;

  for (uint32_t k0 = 0; k0 < passes; k0 += U) {
    u32x2 code[U];
    f32x2 sm[U];
    uint32_t tok[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t k = k0 + u < passes ? k0 + u : passes - 1;
      uint32_t j, kk, run, f;
      fd_divmod(p.dpr, k, j, kk);    // row of tiles of the unit, pass inside the row
      fd_divmod(p.dnf, kk, run, f);
      tok[u] = (tile0 + j * (uint32_t)g.TX + run * (uint32_t)p.rows_q) * (uint32_t)g.F + f + ff;
      code[u] = stream_load<u32x2>(src + ((size_t)f * p.frame_stride + j * row_bytes + run * 512u));
      if (MODE == KVC_Q_PER_TOKEN) {
        const uint32_t tp = tok[u] < n ? tok[u] : n - 1u;  // positions without a token: any pair in bounds
        sm[u] = *(const KVC_GLOBAL f32x2*)(mrow + (size_t)tp * ((uint32_t)g.H * 8u));
      }
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (k0 + u >= passes) continue;  // wave-uniform
      const bool valid = tok[u] < n;
      const uint32_t t = valid ? tok[u] : n - 1u;
      uint64_t off;
      bool ok = valid;
      if (PAGED) {
        uint32_t b, slot;
        fd_divmod(p.dbs, pos0 + t, b, slot);
        const int32_t phys = as_const(p.table)[b];
        const bool in_cache = (uint32_t)phys < (uint32_t)p.num_blocks;
        // an id outside the cache: skip the block's writes and report it (Sec. 3.3.2 placement)
        bad = bad || (valid && !in_cache);
        ok = valid && in_cache;
        off = ((uint64_t)(in_cache ? (uint32_t)phys : 0u) * p.dbs.d + slot) * ((uint32_t)g.C * 2u);
      } else {
        off = (uint64_t)t * (uint64_t)p.ts * 2u;
      }
      if (ok) dequant_store<MODE, DT>(reinterpret_cast<uint16_t*>(obase + off), code[u], sc, mn, sm[u]);
    }
  }
  if (PAGED && bad && e == 0 && p.err) atomicOr(p.err, 1u);
}

// ----------------------------------------------------------------- "lanes" body

template <int MODE, int DT, bool PAGED>
__device__ __forceinline__ void restore_body_lanes(const RestoreParams& p, uint32_t c, uint32_t kind, uint32_t l,
                                                   uint32_t tbi, const uint8_t* fsec, uint32_t ff) {
  constexpr int U = KVC_RESTORE_U;
  const Geo& g = p.g;
  const uint32_t tid = threadIdx.x;
  const uint32_t tsub = fd_div(p.dapt, tid);
  const uint32_t e = (tid - tsub * (uint32_t)g.apt) * 8u;

  const int64_t chunk_first = (int64_t)c * g.T;
  const int64_t left = p.n_tokens - chunk_first;
  const int32_t n = left < (int64_t)g.T ? (int32_t)left : g.T;
  const int32_t ns = p.frame_mode ? (n > (int32_t)ff ? (n - (int32_t)ff + g.F - 1) / g.F : 0) : n;  // token slots, as above
  const int32_t t0 = (int32_t)tbi * p.tb;
  const int32_t t1 = t0 + p.tb < ns ? t0 + p.tb : ns;
  if (t0 >= t1) return;

  uint32_t r, cc;
  tile_pos(g, e, r, cc);
  const uint8_t* fbase = fsec + (r * (uint32_t)g.W + cc);
  const float* mbase = p.meta + (int64_t)c * g.meta_floats + p.moff[kind];
  const uint32_t lm = l - (uint32_t)p.meta_l0;  // layer index inside the pairs that `meta` holds
  float sc[8], mn[8];
  const float* mrow = nullptr;
  if (MODE == KVC_Q_PER_CHANNEL)
    load_channel_pairs(mbase, (int64_t)lm * g.C + e, sc, mn);
  else
    mrow = mbase + 2 * ((int64_t)lm * g.T * g.H + fd_div(g.dD, e));
  uint16_t* obase;
  if (PAGED)
    obase = reinterpret_cast<uint16_t*>(as_const(p.layer_cache)[l]) + (int64_t)kind * p.num_blocks * p.dbs.d * g.C + e;
  else
    obase = p.out + (int64_t)l * p.ls + (int64_t)kind * p.ks + chunk_first * p.ts + e;
  const uint32_t pos0 = (uint32_t)(p.first_token + chunk_first);

  const int32_t step = p.tpp;
  for (int32_t tb0 = t0; tb0 < t1; tb0 += U * step) {
    u32x2 code[U];
    f32x2 sm[U];
    uint16_t* dst[U];
    bool live[U];
    bool bad = false;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t t = tb0 + u * step + (int32_t)tsub;
      live[u] = t < t1;
      const uint32_t tslot = (uint32_t)(live[u] ? t : t1 - 1);
      const uint32_t tc = p.frame_mode ? tslot * (uint32_t)g.F + ff : tslot;
      uint32_t gi, f, ty, tx;
      fd_divmod(g.dF, tc, gi, f);
      fd_divmod(g.dTX, gi, ty, tx);
      code[u] = stream_load<u32x2>(fbase + ((size_t)f * p.frame_stride + ty * p.tile_row_stride + tx * (uint32_t)g.tw));
      if (MODE == KVC_Q_PER_TOKEN) sm[u] = *(const KVC_GLOBAL f32x2*)(mrow + 2 * (int64_t)tc * g.H);
      if (PAGED) {
        uint32_t b, slot;
        fd_divmod(p.dbs, pos0 + tc, b, slot);
        const int32_t phys = as_const(p.table)[b];
        const bool in_cache = (uint32_t)phys < (uint32_t)p.num_blocks;
        bad = bad || (live[u] && !in_cache);
        live[u] = live[u] && in_cache;
        dst[u] = obase + ((int64_t)(in_cache ? phys : 0) * p.dbs.d + slot) * g.C;
      } else {
        dst[u] = obase + (int64_t)tc * p.ts;
      }
    }
    if (PAGED && bad && e == 0 && p.err) atomicOr(p.err, 1u);
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (live[u]) dequant_store<MODE, DT>(dst[u], code[u], sc, mn, sm[u]);
  }
}

// Workgroups are handed to the 8 XCDs round-robin.
//
// Chunk call: a "row" is one (kind, layer), i.e. one region [num_blocks][block][H][D] of a paged
// cache.  The whole chip works on one row at a time; the row's token blocks (over all chunks of the
// call) are cut into 8 contiguous parts, one per XCD, so the workgroups that share a layer's
// per-channel pairs and a run of block-table entries also share an L2, and the writes in flight stay
// inside one region of the cache.
//
// Frame call: units are (frame of the run, plane, block of token slots), each XCD one contiguous range.
constexpr int kBodyLanes = 0, kBodyWaves = 1, kBodyRows = 2;

template <int DT, bool PAGED, int BODY>
__global__ void __launch_bounds__(1024) restore_kernel(const RestoreParams p) {
  const uint32_t xcd = blockIdx.x & 7u, idx = blockIdx.x >> 3;
  uint32_t tbi, l, kind, c, ff = 0;
  const uint8_t* fsec;  // plane of layer l: frame 0 of its group (chunk call) or the one frame (frame call)
  if (p.frame_mode) {
    const uint32_t unit = xcd * p.units_per_xcd + idx;
    if (unit >= p.n_units) return;
    uint32_t rest;
    fd_divmod(p.dtbc, unit, rest, tbi);
    // `frames` holds fm_count consecutive frames, the first being number fm_first of its chunk in
    // the order [kind][layer group][frame of the group]; a frame carries the (up to) three layers
    // of its group, one per plane.
    // A second run of frames (fm_first2, at frames2) may follow the first fm_count1 frames in the same launch.
    uint32_t frel = rest / 3u;
    const uint32_t pl = rest - frel * 3u;
    const uint8_t* run = p.frames;
    uint32_t fno = (uint32_t)p.fm_first + frel;
    if (frel >= (uint32_t)p.fm_count1) {
      frel -= (uint32_t)p.fm_count1;
      fno = (uint32_t)p.fm_first2 + frel;
      run = p.frames2;
    }
    uint32_t q, lg;
    fd_divmod(p.g.dF, fno, q, ff);
    fd_divmod(p.dLG, q, kind, lg);
    l = lg * 3u + pl;
    c = 0;
    if (l >= (uint32_t)p.g.L) return;
    fsec = run + ((int64_t)frel * 3 + pl) * p.g.plane;
  } else {
    uint32_t row, within;
    fd_divmod(p.drpx, idx, row, within);
    const uint32_t u = xcd * p.drpx.d + within;
    if (u >= p.row_units) return;
    fd_divmod(p.dL, row, kind, l);
    fd_divmod(p.dtbc, u, c, tbi);
    const uint32_t lg = l / 3u, pl = l - lg * 3u;
    fsec = p.frames + (int64_t)c * p.g.frame_bytes + (((int64_t)kind * p.g.LG + lg) * p.g.F * 3 + pl) * p.g.plane;
  }
  if (p.g.mode[kind] == KVC_Q_PER_CHANNEL) {
    if (BODY == kBodyRows)
      restore_body_rows<KVC_Q_PER_CHANNEL, DT, PAGED>(p, c, kind, l, tbi, fsec, ff);
    else if (BODY == kBodyWaves)
      restore_body_waves<KVC_Q_PER_CHANNEL, DT, PAGED>(p, c, kind, l, tbi, fsec, ff);
    else
      restore_body_lanes<KVC_Q_PER_CHANNEL, DT, PAGED>(p, c, kind, l, tbi, fsec, ff);
  } else {
    if (BODY == kBodyRows)
      restore_body_rows<KVC_Q_PER_TOKEN, DT, PAGED>(p, c, kind, l, tbi, fsec, ff);
    else if (BODY == kBodyWaves)
      restore_body_waves<KVC_Q_PER_TOKEN, DT, PAGED>(p, c, kind, l, tbi, fsec, ff);
    else
      restore_body_lanes<KVC_Q_PER_TOKEN, DT, PAGED>(p, c, kind, l, tbi, fsec, ff);
  }
}

template <int DT, bool PAGED>
void launch_variant(const RestoreParams& p, int body, dim3 grid, dim3 block, hipStream_t s) {
  if (body == kBodyRows)
    hipLaunchKernelGGL((restore_kernel<DT, PAGED, kBodyRows>), grid, block, 0, s, p);
  else if (body == kBodyWaves)
    hipLaunchKernelGGL((restore_kernel<DT, PAGED, kBodyWaves>), grid, block, 0, s, p);
  else
    hipLaunchKernelGGL((restore_kernel<DT, PAGED, kBodyLanes>), grid, block, 0, s, p);
}

}  // namespace

kvc_status launch_restore(RestoreParams p, bool paged, hipStream_t stream) {
  const Geo& g = p.g;
  if (p.n_tokens <= 0) return KVC_OK;
  if (g.apt > 1024) return KVC_ERR_UNSUPPORTED;
  // threads: a whole number of tokens per pass, about 512 threads
#ifndef KVC_RESTORE_THREADS
#define KVC_RESTORE_THREADS 512
#endif
  const int tpp = g.apt >= KVC_RESTORE_THREADS ? 1 : KVC_RESTORE_THREADS / g.apt;
  const bool waves = g.apt % 64 == 0;
  // The "rows" body: chunk calls on tiles narrower than a 512-byte run whose rows of tiles hold whole runs, when
  // the frames are read over the host link.  (On frames in HBM it is 0.5 % faster than "waves" when the blocks of
  // the cache are in order and 0.4 % slower under a random block table: 1.136 / 1.185 against 1.142 / 1.180 ms.)
  const int q = g.tw < 512 && 512 % g.tw == 0 ? 512 / g.tw : 0;
  const bool rows = p.host_frames && waves && q >= 2 && g.TX % q == 0 && g.th <= 16;
  const int threads = rows ? g.th * 64 : g.apt * tpp;
  const int body = rows ? kBodyRows : waves ? kBodyWaves : kBodyLanes;
  p.rows_body = rows ? 1 : 0;
  if (rows) {
    p.rows_q = q;
    p.rows_lat = 0;
    while ((8 << p.rows_lat) < g.tw) ++p.rows_lat;
    const int nf = p.frame_mode ? 1 : g.F, per_row = nf * (g.TX / q);  // passes one row of tiles takes
    p.dnf = make_fastdiv((uint32_t)nf);
    p.dpr = make_fastdiv((uint32_t)per_row);
    p.rows_trw = per_row >= KVC_RESTORE_U ? 1 : KVC_RESTORE_U / per_row;  // about one round of loads per wave
    p.rows_tile_rows = (int32_t)(((g.T + g.F - 1) / g.F + g.TX - 1) / g.TX);  // rows of tiles that hold tokens
    p.tb = p.rows_trw * g.TX * g.F;  // tokens (chunk call) a workgroup takes
  }
  p.tpp = tpp;
  p.dapt = make_fastdiv((uint32_t)g.apt);
  p.dwpt = make_fastdiv((uint32_t)(waves ? g.apt / 64 : 1));
  if (g.frame_bytes >= (1ll << 32)) return KVC_ERR_UNSUPPORTED;  // offsets inside a chunk section are 32-bit
  p.frame_stride = p.frame_mode ? 0u : (uint32_t)(3 * g.plane);
  if (!p.meta_sliced) {  // `meta` holds whole chunk sections
    p.meta_l0 = 0;
    p.moff[0] = g.meta_off[0];
    p.moff[1] = g.meta_off[1];
  }
  p.tile_row_stride = (uint32_t)g.th * (uint32_t)g.W;
  if (!rows) {
    if (p.tb <= 0) p.tb = waves ? KVC_RESTORE_TB : KVC_RESTORE_TB_LANES;
    if (waves && p.tb > 64 * tpp) p.tb = 64 * tpp;  // one lane per token of a wave
    if (p.tb > g.T) p.tb = g.T;
  }
  p.tbc = (g.T + p.tb - 1) / p.tb;
  p.n_chunks = (int32_t)((p.n_tokens + g.T - 1) / g.T);
  p.dL = make_fastdiv((uint32_t)g.L);
  p.dLG = make_fastdiv((uint32_t)g.LG);
  dim3 grid, block((unsigned)threads);
  if (rows) p.tbc = (p.rows_tile_rows + p.rows_trw - 1) / p.rows_trw;  // units of one (chunk, kind, layer) or plane
  if (p.frame_mode) {
    if (!rows) p.tbc = ((g.T + g.F - 1) / g.F + p.tb - 1) / p.tb;  // slots of one frame
    const int64_t units = (int64_t)p.fm_count * 3 * p.tbc;
    if (units > 0x7fffffff / 8) return KVC_ERR_UNSUPPORTED;
    p.n_units = (uint32_t)units;
    p.units_per_xcd = (p.n_units + 7u) / 8u;
    grid = dim3(p.units_per_xcd * 8u);
  } else {
    const int64_t row_units = (int64_t)p.n_chunks * p.tbc;
    const int64_t per_xcd = (row_units + 7) / 8;
    const int64_t wgs = per_xcd * 8 * 2 * g.L;
    if (wgs > 0x7fffffff) return KVC_ERR_UNSUPPORTED;
    p.row_units = (uint32_t)row_units;
    p.drpx = make_fastdiv((uint32_t)per_xcd);
    grid = dim3((uint32_t)wgs);
  }
  p.dtbc = make_fastdiv((uint32_t)p.tbc);
  if (g.dtype == KVC_F16) {
    if (paged)
      launch_variant<KVC_F16, true>(p, body, grid, block, stream);
    else
      launch_variant<KVC_F16, false>(p, body, grid, block, stream);
  } else {
    if (paged)
      launch_variant<KVC_BF16, true>(p, body, grid, block, stream);
    else
      launch_variant<KVC_BF16, false>(p, body, grid, block, stream);
  }
  return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_RUNTIME;
}

}  // namespace kvc
