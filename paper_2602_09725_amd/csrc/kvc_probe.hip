// Reference streaming kernel for the measurements (not a step of the paper's path): a copy with the
// byte ratio of restore -- 8 bytes read and 16 written per lane, i.e. 1 byte in for 2 bytes out -- whose
// destination can be cut into pieces that land in a caller-given order.  bench.py runs it sequentially
// and with 32 KB pieces (one cache block of the paged workload) in seeded random order, in one-shot
// workgroups of 4 KB and of 32 KB, to show what the part delivers for the access pattern the restore
// kernel is asked for, and uses its sequential form as the copy of known size that the rocprofv3
// FETCH_SIZE / WRITE_SIZE counters are scaled by.  Two switches of the 4 KB shape show why restore cannot
// have that shape's rate: which XCD the eight workgroups of a 32 KB piece run on, and whether a workgroup
// reads its 2 KB in one run or, like the codes of two tokens in a frame (Sec. 3.2.1 step 3, tile (8,128)),
// as 16 lines of 128 bytes 1 KB apart.
#include <hip/hip_runtime.h>

#include "kvc_device.h"
#include "kvc_launch.h"

namespace kvc {

namespace {

// A workgroup moves THREADS * U * 16 bytes of output in one shot: all loads, then all stores.
template <int THREADS, int U>
__global__ void __launch_bounds__(THREADS) expand_kernel(const u32x2* __restrict__ src, u32x4* __restrict__ dst,
                                                         const uint32_t* __restrict__ piece_map, uint32_t log2_vec_per_piece) {
  const size_t base = (size_t)blockIdx.x * THREADS * U;
  const uint32_t t = threadIdx.x;
  u32x2 v[U];
#pragma unroll
  for (int u = 0; u < U; ++u) v[u] = stream_load<u32x2>(src + base + (size_t)u * THREADS + t);
#pragma unroll
  for (int u = 0; u < U; ++u) {
    const size_t j = base + (size_t)u * THREADS + t;  // 16-byte vector of the output, in source order
    size_t d = j;
    if (piece_map) {
      const size_t piece = j >> log2_vec_per_piece, off = j & (((size_t)1 << log2_vec_per_piece) - 1);
      d = ((size_t)piece_map[piece] << log2_vec_per_piece) + off;
    }
    stream_store<u32x4>(dst + d, u32x4{v[u].x, v[u].y, v[u].x ^ v[u].y, (uint32_t)j});
  }
}

// The 4 KB shape with the two switches.  Workgroups are handed to the 8 XCDs round-robin: with ONE_XCD the
// units 8k .. 8k+7 (one 32 KB piece) go to one XCD instead of one to each; with LINES unit 8k+m reads the lines
// m, m+8, .. m+120 of the 16 KB that its group of 8 units reads together.
template <bool ONE_XCD, bool LINES>
__global__ void __launch_bounds__(256) expand_shaped_kernel(const u32x2* __restrict__ src, u32x4* __restrict__ dst,
                                                            const uint32_t* __restrict__ piece_map, uint32_t log2_vec_per_piece) {
  const uint32_t b = blockIdx.x, t = threadIdx.x;
  const uint32_t unit = ONE_XCD ? (b & 7u) * (gridDim.x >> 3) + (b >> 3) : b;
  const size_t j = (size_t)unit * 256 + t;  // 16-byte vector of the output, in source order
  size_t sv = j;                            // 8-byte vector of the source
  if (LINES) sv = (size_t)(unit >> 3) * 2048 + (size_t)((unit & 7u) + 8u * (t >> 4)) * 16u + (t & 15u);
  const u32x2 v = stream_load<u32x2>(src + sv);
  size_t d = j;
  if (piece_map) {
    const size_t piece = j >> log2_vec_per_piece, off = j & (((size_t)1 << log2_vec_per_piece) - 1);
    d = ((size_t)piece_map[piece] << log2_vec_per_piece) + off;
  }
  stream_store<u32x4>(dst + d, u32x4{v.x, v.y, v.x ^ v.y, (uint32_t)sv});
}

}  // namespace

kvc_status launch_probe_expand(const void* src, void* dst, size_t out_bytes, const uint32_t* piece_map, uint32_t log2_piece,
                               int32_t wg_bytes, int32_t shape, hipStream_t stream) {
  const uint32_t lg = log2_piece - 4;  // 16-byte vectors per piece
  const size_t wgs = out_bytes / (size_t)wg_bytes;
  if (wgs == 0) return KVC_OK;
  if (wgs > 0x7fffffff) return KVC_ERR_UNSUPPORTED;
  const dim3 grid((uint32_t)wgs);
  const u32x2* s = static_cast<const u32x2*>(src);
  u32x4* d = static_cast<u32x4*>(dst);
  if (shape != 0) {  // 4 KB workgroups, a multiple of 8 of them (checked by the caller)
    const bool one_xcd = (shape & KVC_PROBE_ONE_XCD_PER_PIECE) != 0, lines = (shape & KVC_PROBE_LINE_READS) != 0;
    if (one_xcd && lines)
      hipLaunchKernelGGL((expand_shaped_kernel<true, true>), grid, dim3(256), 0, stream, s, d, piece_map, lg);
    else if (one_xcd)
      hipLaunchKernelGGL((expand_shaped_kernel<true, false>), grid, dim3(256), 0, stream, s, d, piece_map, lg);
    else
      hipLaunchKernelGGL((expand_shaped_kernel<false, true>), grid, dim3(256), 0, stream, s, d, piece_map, lg);
  } else if (wg_bytes == 4096) {
    hipLaunchKernelGGL((expand_kernel<256, 1>), grid, dim3(256), 0, stream, s, d, piece_map, lg);
  } else {
    hipLaunchKernelGGL((expand_kernel<512, 4>), grid, dim3(512), 0, stream, s, d, piece_map, lg);
  }
  return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_RUNTIME;
}

}  // namespace kvc
