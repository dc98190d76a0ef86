// Codec-free score of a packed chunk for the intra-frame tiling search (Sec. 3.2.2).
//
// The paper ranks the candidate tilings by the size of the encoded video.  Without an encoder
// the search here ranks them by what a predictive coder would have to store: histograms of the
// residuals of the 8-bit codes against the predictors a video codec has -- the pixel to the left,
// the pixel above, the same pixel of the previous frame (Sec. 3.2.1 step 3 puts the next token
// there), and that temporal residual after its own left / upper neighbour.  The kernel only counts;
// entropies and the cost in bits are host arithmetic (kvc_proxy_cost_bits).
//
// One workgroup per plane sequence (chunk, kind, layer): it owns the five histograms of its stream,
// so the result needs no atomics in global memory and no cleared buffer.  Every frame byte is read
// from HBM once: a thread walks down a column, so the row above is its own previous read (a cache hit),
// and the byte to the left sits in the line it is reading anyway.  Counting is done with LDS
// atomics on 16 copies of the histograms (lanes spread over the copies, so that equal residuals in one
// wave seldom meet in one counter), which is what bounds the kernel: five counter updates per pixel
// against one byte of HBM traffic; with the counting switched off the same loop runs in a third of the time.
#include <hip/hip_runtime.h>

#include "kvc_device.h"
#include "kvc_launch.h"

namespace kvc {

namespace {

constexpr int kScoreThreads = 512;
constexpr int kCopies = 16;  // copies of each histogram in LDS: 80 KB of the CU's 160 KB (4 copies: 2.1 ms, 16: 1.36 ms)

// a - b on each of the four bytes of a word, modulo 256
__device__ __forceinline__ uint32_t sub_bytes(uint32_t a, uint32_t b) {
  const uint32_t top = 0x80808080u;
  return ((a | top) - (b & ~top)) ^ ((a ^ ~b) & top);
}

// The 8 pixels one position to the left of v's: v shifted up by a byte, `left` (in bits 31..24) entering.
__device__ __forceinline__ u32x2 left_of(u32x2 v, uint32_t left) {
  u32x2 o;
  o.x = __builtin_amdgcn_alignbyte(v.x, left, 3);
  o.y = __builtin_amdgcn_alignbyte(v.y, v.x, 3);
  return o;
}

__device__ __forceinline__ u32x2 sub_bytes(u32x2 a, u32x2 b) { return u32x2{sub_bytes(a.x, b.x), sub_bytes(a.y, b.y)}; }

__device__ __forceinline__ void count8(uint32_t (*h)[kCopies], u32x2 v, uint32_t copy) {
#pragma unroll
  for (int i = 0; i < 8; ++i) {
    const uint32_t w = i < 4 ? v.x : v.y;
    atomicAdd(&h[(w >> (8 * (i & 3))) & 0xffu][copy], 1u);
  }
}

__global__ void __launch_bounds__(kScoreThreads) residual_hist_kernel(const ScoreParams p) {
  __shared__ uint32_t hist[KVC_N_RESIDUALS][256][kCopies];
  const Geo& g = p.g;
  const uint32_t tid = threadIdx.x;
  for (uint32_t i = tid; i < KVC_N_RESIDUALS * 256u * kCopies; i += kScoreThreads) (&hist[0][0][0])[i] = 0u;
  __syncthreads();

  const uint32_t s = blockIdx.x;  // stream = (chunk, kind, layer)
  uint32_t ck, l;
  fd_divmod(p.dL, s, ck, l);
  const uint32_t kind = ck & 1u, c = ck >> 1;
  const uint32_t lg = l / 3u, pl = l - lg * 3u;
  const uint8_t* base = p.frames + (int64_t)c * g.frame_bytes + (((int64_t)kind * g.LG + lg) * g.F * 3 + pl) * g.plane;
  const int64_t frame_stride = 3 * g.plane;
  const uint32_t W = (uint32_t)g.W, per_row = W / 8u;
  const uint32_t copy = tid & (kCopies - 1);

  // A thread walks down a column of 8-pixel pieces, so the row above is what it read itself one step earlier (a
  // cache hit, never a second miss in flight for the same line).  Rows narrower than the workgroup are cut into
  // bands of rows worked side by side; wider rows are taken in blocks of kScoreThreads columns.
  const uint32_t cols = per_row < (uint32_t)kScoreThreads ? per_row : (uint32_t)kScoreThreads;
  const uint32_t bands = (uint32_t)kScoreThreads / cols;
  const uint32_t band = tid / cols, col0 = tid - band * cols;
  const uint32_t rows_per_band = ((uint32_t)g.Hp + bands - 1u) / bands;
  const uint32_t y0 = band * rows_per_band;
  uint32_t y1 = y0 + rows_per_band;
  y1 = y1 < (uint32_t)g.Hp ? y1 : (uint32_t)g.Hp;
  for (uint32_t cb = col0; band < bands && cb < per_row; cb += cols)
  for (uint32_t y = y0; y < y1; ++y) {
    const uint32_t q = y * per_row + cb;  // piece = 8 pixels of a row; rows are contiguous
    const bool has_up = y > 0u, has_left = q - y * per_row > 0u;
    u32x2 prev{0u, 0u}, prev_up{0u, 0u};
    uint32_t prev_left = 0u;
    for (uint32_t f = 0; f < (uint32_t)g.F; ++f) {
      const uint8_t* px = base + (int64_t)f * frame_stride + (size_t)q * 8u;
      const u32x2 cur = *(const KVC_GLOBAL u32x2*)px;  // cached: the next row reads it again as its upper neighbour
      const u32x2 up = has_up ? *(const KVC_GLOBAL u32x2*)(px - W) : u32x2{0u, 0u};
      const uint32_t left = has_left ? (uint32_t)(*(const KVC_GLOBAL uint8_t*)(px - 1)) << 24 : 0u;
      count8(hist[KVC_RES_LEFT], sub_bytes(cur, left_of(cur, left)), copy);
      count8(hist[KVC_RES_UP], sub_bytes(cur, up), copy);
      if (f > 0u) {
        const u32x2 t = sub_bytes(cur, prev);
        const uint32_t t_left = sub_bytes(left, prev_left);  // the temporal residual of the pixel to the left
        count8(hist[KVC_RES_TIME], t, copy);
        count8(hist[KVC_RES_TIME_LEFT], sub_bytes(t, left_of(t, t_left)), copy);
        count8(hist[KVC_RES_TIME_UP], sub_bytes(t, sub_bytes(up, prev_up)), copy);
      }
      prev = cur;
      prev_up = up;
      prev_left = left;
    }
  }
  __syncthreads();
  uint64_t* out = p.hist + (size_t)s * (KVC_N_RESIDUALS * 256);
  for (uint32_t i = tid; i < KVC_N_RESIDUALS * 256u; i += kScoreThreads) {
    const uint32_t* hc = &(&hist[0][0][0])[i * kCopies];
    uint64_t n = 0;
#pragma unroll
    for (int k = 0; k < kCopies; ++k) n += hc[k];
    out[i] = n;
  }
}

}  // namespace

kvc_status launch_residual_histograms(ScoreParams p, hipStream_t stream) {
  const Geo& g = p.g;
  if (p.n_chunks <= 0) return KVC_OK;
  if ((int64_t)g.F * g.plane >= (1ll << 32)) return KVC_ERR_UNSUPPORTED;  // 32-bit counters per stream
  const int64_t streams = (int64_t)p.n_chunks * 2 * g.L;
  if (streams > 0x7fffffff) return KVC_ERR_UNSUPPORTED;
  p.dL = make_fastdiv((uint32_t)g.L);
  hipLaunchKernelGGL(residual_hist_kernel, dim3((uint32_t)streams), dim3(kScoreThreads), 0, stream, p);
  return hipGetLastError() == hipSuccess ? KVC_OK : KVC_ERR_RUNTIME;
}

}  // namespace kvc
