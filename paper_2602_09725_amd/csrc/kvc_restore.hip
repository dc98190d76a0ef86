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
// contiguous block of tokens of one (chunk, kind, layer); thread i keeps atom
// i % (C/8) for the whole block, so
//   - a wave's load covers 512 contiguous code bytes and its store 1024
//     contiguous output bytes (full cache lines both ways),
//   - per-channel scale/min of the thread's 8 channels are loaded once and stay
//     in 16 VGPRs,
//   - when C/8 is a multiple of 64 the token index is wave-uniform and all
//     index arithmetic (frame, tile position, cache slot, block-table lookup)
//     runs on the scalar unit.
// A contiguous block of tokens touches F frames at TX-adjacent tile positions,
// i.e. a few contiguous runs of th rows in each of F planes (Sec. 3.2.1 step 3),
// so both sides of the copy stay DRAM-page friendly.
#include <hip/hip_runtime.h>

#include "kvc_device.h"
#include "kvc_launch.h"

namespace kvc {

#ifndef KVC_RESTORE_U
#define KVC_RESTORE_U 8  // token passes in flight per thread
#endif

namespace {

template <int MODE, int DT, bool PAGED, bool UNIFORM>
__device__ __forceinline__ void restore_body(const RestoreParams& p, uint32_t c, uint32_t kind, uint32_t l,
                                             uint32_t tbi) {
  constexpr int U = KVC_RESTORE_U;
  const Geo& g = p.g;
  const uint32_t tid = threadIdx.x;
  uint32_t tsub = fd_div(p.dapt, tid);
  const uint32_t ca = tid - tsub * (uint32_t)g.apt;
  if (UNIFORM) tsub = wave_uniform(tsub);
  const uint32_t e = ca * 8u;

  const int64_t chunk_first = (int64_t)c * g.T;
  const int64_t left = p.n_tokens - chunk_first;
  const int32_t n = left < (int64_t)g.T ? (int32_t)left : g.T;  // valid tokens of this chunk
  const int32_t t0 = (int32_t)tbi * p.tb;
  const int32_t t1 = t0 + p.tb < n ? t0 + p.tb : n;
  if (t0 >= t1) return;

  // intra-frame layout: element e of the token -> (row, column) of its tile
  uint32_t r, cc;
  fd_divmod(g.dtw, e, r, cc);
  const uint32_t lg = l / 3u, pl = l - lg * 3u;
  const uint8_t* fbase = p.frames + (int64_t)c * g.frame_bytes +
                         (((int64_t)kind * g.LG + lg) * g.F * 3 + pl) * g.plane + (r * (uint32_t)g.W + cc);
  const float* mbase = p.meta + (int64_t)c * g.meta_floats + g.meta_off[kind];

  float sc[8], mn[8];
  const float* mrow = nullptr;
  if (MODE == KVC_Q_PER_CHANNEL) {
    const KVC_GLOBAL f32x2* mp = (const KVC_GLOBAL f32x2*)(mbase + 2 * ((int64_t)l * g.C + e));
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const f32x2 v = mp[i];
      sc[i] = v.x;
      mn[i] = v.y;
    }
  } else {
    const uint32_t h = fd_div(g.dD, e);
    mrow = mbase + 2 * ((int64_t)l * g.T * g.H + h);
  }

  uint16_t* obase;
  if (PAGED) {
    obase = reinterpret_cast<uint16_t*>(as_const(p.layer_cache)[l]) + (int64_t)kind * p.num_blocks * p.dbs.d * g.C + e;
  } else {
    obase = p.out + (int64_t)l * p.ls + (int64_t)kind * p.ks + chunk_first * p.ts + e;
  }
  const uint32_t pos0 = (uint32_t)(p.first_token + chunk_first);  // sequence position of the chunk's token 0

  const int32_t step = p.tpp;
  for (int32_t tb0 = t0; tb0 < t1; tb0 += U * step) {
    u32x2 code[U];
    f32x2 sm[U];
    uint16_t* dst[U];
    bool live[U];      // wave-uniform when the token index is
    uint32_t slot[U];  // paged: slot inside the block
    int32_t phys[U];   // paged: physical block id
    // 1) all streaming loads of the batch are issued before anything waits
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int32_t t = tb0 + u * step + (int32_t)tsub;
      live[u] = t < t1;
      const uint32_t tc = (uint32_t)(live[u] ? t : t1 - 1);  // clamp: the load stays in bounds, the store is skipped
      // inter-frame layout: token -> (frame of its group, tile position of its group)
      uint32_t gi, f, ty, tx;
      fd_divmod(g.dF, tc, gi, f);
      fd_divmod(g.dTX, gi, ty, tx);
      const uint8_t* src = fbase + (int64_t)f * 3 * g.plane + ((int64_t)ty * g.th * g.W + tx * (uint32_t)g.tw);
      code[u] = stream_load<u32x2>(src);
      if (MODE == KVC_Q_PER_TOKEN) sm[u] = *(const KVC_GLOBAL f32x2*)(mrow + 2 * (int64_t)tc * g.H);
      if (PAGED) {
        uint32_t b;
        fd_divmod(p.dbs, pos0 + tc, b, slot[u]);
        phys[u] = as_const(p.table)[b];
      } else {
        dst[u] = obase + (int64_t)tc * p.ts;
      }
    }
    // 2) placement (Sec. 3.3.2: preallocated slots of the paged memory)
    if (PAGED) {
      bool bad = false;
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const bool in_cache = (uint32_t)phys[u] < (uint32_t)p.num_blocks;
        bad = bad || (live[u] && !in_cache);
        live[u] = live[u] && in_cache;  // an id outside the cache: skip the block's writes
        dst[u] = obase + ((int64_t)(in_cache ? phys[u] : 0) * p.dbs.d + slot[u]) * g.C;
      }
      if (bad && ca == 0 && p.err) atomicOr(p.err, 1u);  // ... and report it
    }
    // 3) dequantize and store
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (!live[u]) continue;
      float x[8];
#pragma unroll
      for (int i = 0; i < 8; ++i) {
        const uint32_t w = i < 4 ? code[u].x : code[u].y;
        const float q = (float)((w >> (8 * (i & 3))) & 0xffu);
        x[i] = MODE == KVC_Q_PER_CHANNEL ? __builtin_fmaf(q, sc[i], mn[i]) : __builtin_fmaf(q, sm[u].x, sm[u].y);
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
      stream_store<u32x4>(dst[u], o);
    }
  }
}

template <int DT, bool PAGED, bool UNIFORM>
__global__ void __launch_bounds__(1024) restore_kernel(const RestoreParams p) {
  // Workgroups are handed to the 8 XCDs round-robin.  Give each XCD one
  // contiguous range of units so that the workgroups sharing a layer's
  // per-channel scale/min and block-table entries also share an L2.
  const uint32_t unit = (blockIdx.x & 7u) * p.units_per_xcd + (blockIdx.x >> 3);
  if (unit >= p.n_units) return;
  uint32_t u = unit;
  const uint32_t tbi = u % (uint32_t)p.tbc;
  u /= (uint32_t)p.tbc;
  const uint32_t l = u % (uint32_t)p.g.L;
  u /= (uint32_t)p.g.L;
  const uint32_t kind = u & 1u;
  const uint32_t c = u >> 1;
  if (p.g.mode[kind] == KVC_Q_PER_CHANNEL)
    restore_body<KVC_Q_PER_CHANNEL, DT, PAGED, UNIFORM>(p, c, kind, l, tbi);
  else
    restore_body<KVC_Q_PER_TOKEN, DT, PAGED, UNIFORM>(p, c, kind, l, tbi);
}

template <int DT, bool PAGED>
void launch_variant(const RestoreParams& p, bool uniform, dim3 grid, dim3 block, hipStream_t s) {
  if (uniform)
    hipLaunchKernelGGL((restore_kernel<DT, PAGED, true>), grid, block, 0, s, p);
  else
    hipLaunchKernelGGL((restore_kernel<DT, PAGED, false>), grid, block, 0, s, p);
}

}  // namespace

kvc_status launch_restore(RestoreParams p, bool paged, hipStream_t stream) {
  const Geo& g = p.g;
  if (p.n_tokens <= 0) return KVC_OK;
  // threads: a whole number of tokens per pass, about 256 threads
  if (g.apt > 1024) return KVC_ERR_UNSUPPORTED;
  const int tpp = g.apt >= 256 ? 1 : 256 / g.apt;
  const int threads = g.apt * tpp;
  p.tpp = tpp;
  p.dapt = make_fastdiv((uint32_t)g.apt);
  if (p.tb <= 0) {
#ifdef KVC_RESTORE_TB
    p.tb = KVC_RESTORE_TB;
#else
    p.tb = 128;
#endif
  }
  if (p.tb > g.T) p.tb = g.T;
  p.tbc = (g.T + p.tb - 1) / p.tb;
  p.n_chunks = (int32_t)((p.n_tokens + g.T - 1) / g.T);
  const int64_t units = (int64_t)p.n_chunks * 2 * g.L * p.tbc;
  if (units > 0x7fffffff / 8) return KVC_ERR_UNSUPPORTED;
  p.n_units = (uint32_t)units;
  p.units_per_xcd = (p.n_units + 7u) / 8u;
  const dim3 grid(p.units_per_xcd * 8u), block((unsigned)threads);
  const bool uniform = g.apt % 64 == 0;
  if (g.dtype == KVC_F16) {
    if (paged)
      launch_variant<KVC_F16, true>(p, uniform, grid, block, stream);
    else
      launch_variant<KVC_F16, false>(p, uniform, grid, block, stream);
  } else {
    if (paged)
      launch_variant<KVC_BF16, true>(p, uniform, grid, block, stream);
    else
      launch_variant<KVC_BF16, false>(p, uniform, grid, block, stream);
  }
  return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_RUNTIME;
}

}  // namespace kvc
