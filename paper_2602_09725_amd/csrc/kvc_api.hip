// Host layer of libkvc: argument validation, derived geometry, the C ABI of
// include/kvc.h and the two-stream fetch pipeline.
#include <hip/hip_runtime.h>

#include <limits.h>
#include <math.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "kvc_launch.h"

namespace kvc {

namespace {

int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

bool aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

kvc_status check_layout(const kvc_layout* lo) {
  if (!lo) return KVC_ERR_INVALID_ARG;
  if (lo->struct_size != sizeof(kvc_layout) || lo->abi_version != KVC_ABI_VERSION) return KVC_ERR_INVALID_ARG;
  if (lo->num_layers < 1 || lo->num_kv_heads < 1 || lo->head_dim < 1 || lo->chunk_tokens < 1) return KVC_ERR_INVALID_ARG;
  if (lo->tile_h < 1 || lo->tile_w < 1 || lo->tiles_x < 1 || lo->tiles_y < 1) return KVC_ERR_INVALID_ARG;
  if ((int64_t)lo->tile_h * lo->tile_w != (int64_t)lo->num_kv_heads * lo->head_dim) return KVC_ERR_INVALID_ARG;
  if (lo->tile_seg < 0) return KVC_ERR_INVALID_ARG;
  if (lo->tile_seg > 0) {  // Sec. 3.2.2: head_num = h1 * h2, head_dim = d1 * d2, tile = (h1 * d1, h2 * d2)
    const int32_t d2 = lo->tile_seg;
    if (lo->head_dim % d2 != 0 || lo->tile_w % d2 != 0) return KVC_ERR_INVALID_ARG;
    const int32_t h2 = lo->tile_w / d2;
    if (lo->num_kv_heads % h2 != 0) return KVC_ERR_INVALID_ARG;
    if ((int64_t)(lo->num_kv_heads / h2) * (lo->head_dim / d2) != lo->tile_h) return KVC_ERR_INVALID_ARG;
  }
  if (lo->dtype != KVC_F16 && lo->dtype != KVC_BF16) return KVC_ERR_INVALID_ARG;
  if (lo->k_mode != KVC_Q_PER_CHANNEL && lo->k_mode != KVC_Q_PER_TOKEN) return KVC_ERR_INVALID_ARG;
  if (lo->v_mode != KVC_Q_PER_CHANNEL && lo->v_mode != KVC_Q_PER_TOKEN) return KVC_ERR_INVALID_ARG;
  // sizes the 32-bit in-plane arithmetic of the kernels can hold
  const int64_t C = (int64_t)lo->num_kv_heads * lo->head_dim;
  const int64_t G = (int64_t)lo->tiles_x * lo->tiles_y;
  const int64_t F = ceil_div(lo->chunk_tokens, G);
  if (C > (1 << 20) || G > (1 << 28) || F * G >= (1ll << 30) || G * C >= (1ll << 31)) return KVC_ERR_UNSUPPORTED;
  if ((int64_t)lo->num_layers > (1 << 20) || (int64_t)lo->chunk_tokens * lo->num_kv_heads >= (1ll << 31))
    return KVC_ERR_UNSUPPORTED;
  return KVC_OK;
}

hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

// Whether p is host memory that is mapped into the device, so that a kernel reads it over the host link.
// (A pointer the runtime does not know leaves an error behind, which is cleared: it is not this call's to report.)
bool in_host_memory(const void* p) {
  hipPointerAttribute_t a;
  if (hipPointerGetAttributes(&a, p) != hipSuccess) {
    (void)hipGetLastError();
    return false;
  }
  return a.type == hipMemoryTypeHost;
}

// Entropy in bits per symbol of a 256-bin histogram (0 for an empty one).
double histogram_entropy(const uint64_t* bins) {
  double n = 0.0;
  for (int i = 0; i < 256; ++i) n += (double)bins[i];
  if (n == 0.0) return 0.0;
  double h = 0.0;
  for (int i = 0; i < 256; ++i)
    if (bins[i]) {
      const double q = (double)bins[i] / n;
      h -= q * log2(q);
    }
  return h;
}

// Lowest index at which cost(i), i in [0, n), is smallest.
template <typename Cost>
int32_t first_argmin(int32_t n, Cost cost) {
  int32_t at = 0;
  double least = cost(0);
  for (int32_t i = 1; i < n; ++i) {
    const double c = cost(i);
    if (c < least) {
      least = c;
      at = i;
    }
  }
  return at;
}

kvc_status check_strides(const kvc_strides& s) {
  if (s.layer_stride < 0 || s.kv_stride < 0 || s.token_stride < 0) return KVC_ERR_INVALID_ARG;
  if ((s.layer_stride | s.kv_stride | s.token_stride) & 7) return KVC_ERR_INVALID_ARG;
  return KVC_OK;
}

}  // namespace

kvc_status make_geo(const kvc_layout* lo, Geo* g) {
  const kvc_status st = check_layout(lo);
  if (st != KVC_OK) return st;
  if (lo->head_dim % 8 != 0 || lo->tile_w % 8 != 0 || lo->tile_seg % 8 != 0) return KVC_ERR_UNSUPPORTED;
  g->L = lo->num_layers;
  g->H = lo->num_kv_heads;
  g->D = lo->head_dim;
  g->C = g->H * g->D;
  g->T = lo->chunk_tokens;
  g->th = lo->tile_h;
  g->tw = lo->tile_w;
  g->TX = lo->tiles_x;
  g->TY = lo->tiles_y;
  g->G = g->TX * g->TY;
  g->F = (int32_t)ceil_div(g->T, g->G);
  g->FG = g->F * g->G;
  g->LG = (int32_t)ceil_div(g->L, 3);
  g->W = g->TX * g->tw;
  g->Hp = g->TY * g->th;
  g->apt = g->C / 8;
  g->dtype = lo->dtype;
  g->mode[0] = lo->k_mode;
  g->mode[1] = lo->v_mode;
  g->plane = (int64_t)g->Hp * g->W;
  g->frame_bytes = 2ll * g->LG * g->F * 3 * g->plane;
  int64_t pairs[2];
  for (int k = 0; k < 2; ++k)
    pairs[k] = g->mode[k] == KVC_Q_PER_CHANNEL ? (int64_t)g->L * g->C : (int64_t)g->L * g->T * g->H;
  g->meta_off[0] = 0;
  g->meta_off[1] = 2 * pairs[0];
  g->meta_floats = 2 * (pairs[0] + pairs[1]);
  g->dF = make_fastdiv((uint32_t)g->F);
  g->dTX = make_fastdiv((uint32_t)g->TX);
  g->dtw = make_fastdiv((uint32_t)g->tw);
  g->dD = make_fastdiv((uint32_t)g->D);
  g->seg = lo->tile_seg;
  g->d1 = g->seg ? g->D / g->seg : 1;
  g->dseg = make_fastdiv((uint32_t)(g->seg ? g->seg : 1));
  g->dh2 = make_fastdiv((uint32_t)(g->seg ? g->tw / g->seg : 1));
  return KVC_OK;
}

}  // namespace kvc

using namespace kvc;

extern "C" {

const char* kvc_status_str(kvc_status status) {
  switch (status) {
    case KVC_OK: return "ok";
    case KVC_ERR_INVALID_ARG: return "invalid argument";
    case KVC_ERR_UNSUPPORTED: return "unsupported layout or size";
    case KVC_ERR_BUFFER_TOO_SMALL: return "buffer too small";
    case KVC_ERR_RUNTIME: return "HIP runtime error";
  }
  return "unknown status";
}

#ifndef KVC_BUILD_ID
#define KVC_BUILD_ID "unknown"
#endif
static const char build_tag[] = "kvc-build-id:" KVC_BUILD_ID;  // also found by scanning the file
const char* kvc_build_id(void) { return build_tag + 13; }

kvc_status kvc_layout_validate(const kvc_layout* layout) { return check_layout(layout); }

kvc_status kvc_chunk_sizes(const kvc_layout* layout, size_t* frame_bytes, size_t* meta_bytes,
                           int32_t* frames_per_group) {
  const kvc_status st = check_layout(layout);
  if (st != KVC_OK) return st;
  const int64_t C = (int64_t)layout->num_kv_heads * layout->head_dim;
  const int64_t G = (int64_t)layout->tiles_x * layout->tiles_y;
  const int64_t F = ceil_div(layout->chunk_tokens, G);
  const int64_t LG = ceil_div(layout->num_layers, 3);
  int64_t pairs = 0;
  const int modes[2] = {layout->k_mode, layout->v_mode};
  for (int k = 0; k < 2; ++k)
    pairs += modes[k] == KVC_Q_PER_CHANNEL ? (int64_t)layout->num_layers * C
                                           : (int64_t)layout->num_layers * layout->chunk_tokens * layout->num_kv_heads;
  if (frame_bytes) *frame_bytes = (size_t)(2 * LG * F * 3 * G * C);
  if (meta_bytes) *meta_bytes = (size_t)(8 * pairs);
  if (frames_per_group) *frames_per_group = (int32_t)F;
  return KVC_OK;
}

size_t kvc_blob_meta_offset(const kvc_layout* layout) {
  size_t fb = 0;
  if (kvc_chunk_sizes(layout, &fb, nullptr, nullptr) != KVC_OK) return 0;
  return (fb + 255) & ~(size_t)255;
}

kvc_status kvc_pack(const kvc_layout* layout, const void* kv, kvc_strides strides, int64_t n_tokens, uint8_t* frames,
                    size_t frames_cap, void* meta, size_t meta_cap, void* stream) {
  PackParams p{};
  kvc_status st = make_geo(layout, &p.g);
  if (st != KVC_OK) return st;
  if (n_tokens < 0 || n_tokens >= (1ll << 31)) return KVC_ERR_INVALID_ARG;
  if (n_tokens == 0) return KVC_OK;
  if (!kv || !frames || !meta) return KVC_ERR_INVALID_ARG;
  if ((st = check_strides(strides)) != KVC_OK) return st;
  if (!aligned(kv, 16) || !aligned(frames, 16) || !aligned(meta, 8)) return KVC_ERR_INVALID_ARG;
  if (strides.token_stride < p.g.C) return KVC_ERR_INVALID_ARG;
  const int64_t n_chunks = ceil_div(n_tokens, p.g.T);
  if ((uint64_t)(n_chunks * p.g.frame_bytes) > frames_cap) return KVC_ERR_BUFFER_TOO_SMALL;
  if ((uint64_t)(n_chunks * p.g.meta_floats * 4) > meta_cap) return KVC_ERR_BUFFER_TOO_SMALL;
  p.kv = static_cast<const uint16_t*>(kv);
  p.ls = strides.layer_stride;
  p.ks = strides.kv_stride;
  p.ts = strides.token_stride;
  p.n_tokens = n_tokens;
  p.frames = frames;
  p.meta = static_cast<float*>(meta);
  return launch_pack(p, as_stream(stream));
}

kvc_status kvc_pack_plan(const kvc_layout* layout, kvc_strides strides, int32_t* resident, int32_t* threads) {
  PackParams p{};
  kvc_status st = make_geo(layout, &p.g);
  if (st != KVC_OK) return st;
  if ((st = check_strides(strides)) != KVC_OK) return st;
  if (strides.token_stride < p.g.C) return KVC_ERR_INVALID_ARG;
  p.ls = strides.layer_stride;
  p.ks = strides.kv_stride;
  p.ts = strides.token_stride;
  p.n_tokens = p.g.T;
  int th = 0;
  if ((st = plan_pack(p, &th)) != KVC_OK) return st;
  if (resident) *resident = p.resident;
  if (threads) *threads = th;
  return KVC_OK;
}

kvc_status kvc_restore(const kvc_layout* layout, const uint8_t* frames, const void* meta, int64_t n_tokens,
                       void* kv_out, kvc_strides strides, void* stream) {
  RestoreParams p{};
  kvc_status st = make_geo(layout, &p.g);
  if (st != KVC_OK) return st;
  if (n_tokens < 0 || n_tokens >= (1ll << 31)) return KVC_ERR_INVALID_ARG;
  if (n_tokens == 0) return KVC_OK;
  if (!kv_out || !frames || !meta) return KVC_ERR_INVALID_ARG;
  if ((st = check_strides(strides)) != KVC_OK) return st;
  if (!aligned(kv_out, 16) || !aligned(frames, 16) || !aligned(meta, 8)) return KVC_ERR_INVALID_ARG;
  if (strides.token_stride < p.g.C) return KVC_ERR_INVALID_ARG;
  p.frames = frames;
  p.meta = static_cast<const float*>(meta);
  p.n_tokens = n_tokens;
  p.out = static_cast<uint16_t*>(kv_out);
  p.ls = strides.layer_stride;
  p.ks = strides.kv_stride;
  p.ts = strides.token_stride;
  p.dbs = make_fastdiv(1);
  p.host_frames = in_host_memory(p.frames);
  return launch_restore(p, false, as_stream(stream));
}

namespace {

// Argument checks shared by kvc_restore_paged and kvc_fetch_pipeline.
kvc_status fill_paged(RestoreParams& p, int64_t first_token, int64_t n_tokens, void* const* d_layer_cache,
                      int64_t num_blocks, int32_t block_size, const int32_t* d_block_table, int64_t table_len,
                      uint32_t* d_err) {
  if (n_tokens < 0 || first_token < 0 || first_token + n_tokens >= (1ll << 31)) return KVC_ERR_INVALID_ARG;
  if (first_token % p.g.T != 0) return KVC_ERR_INVALID_ARG;
  if (num_blocks < 1 || num_blocks >= (1ll << 31) || block_size < 1 || table_len < 0) return KVC_ERR_INVALID_ARG;
  if (!d_layer_cache || !d_block_table) return KVC_ERR_INVALID_ARG;
  if (table_len * block_size < first_token + n_tokens) return KVC_ERR_INVALID_ARG;
  if (d_err && !aligned(d_err, 4)) return KVC_ERR_INVALID_ARG;
  p.layer_cache = d_layer_cache;
  p.table = d_block_table;
  p.num_blocks = num_blocks;
  p.dbs = make_fastdiv((uint32_t)block_size);
  p.first_token = first_token;
  p.err = d_err;
  p.n_tokens = n_tokens;
  return KVC_OK;
}

}  // namespace

kvc_status kvc_restore_paged(const kvc_layout* layout, const uint8_t* frames, const void* meta, int64_t first_token,
                             int64_t n_tokens, void* const* d_layer_cache, int64_t num_blocks, int32_t block_size,
                             const int32_t* d_block_table, int64_t table_len, uint32_t* d_err, void* stream) {
  RestoreParams p{};
  kvc_status st = make_geo(layout, &p.g);
  if (st != KVC_OK) return st;
  if ((st = fill_paged(p, first_token, n_tokens, d_layer_cache, num_blocks, block_size, d_block_table, table_len,
                       d_err)) != KVC_OK)
    return st;
  if (n_tokens == 0) return KVC_OK;
  if (!frames || !meta) return KVC_ERR_INVALID_ARG;
  if (!aligned(frames, 16) || !aligned(meta, 8)) return KVC_ERR_INVALID_ARG;
  p.frames = frames;
  p.meta = static_cast<const float*>(meta);
  p.host_frames = in_host_memory(p.frames);
  return launch_restore(p, true, as_stream(stream));
}

size_t kvc_residual_histograms_size(const kvc_layout* layout, int64_t n_chunks) {
  if (check_layout(layout) != KVC_OK || n_chunks < 0 || n_chunks > (1 << 24)) return (size_t)-1;
  return (size_t)n_chunks * 2 * (size_t)layout->num_layers * KVC_N_RESIDUALS * 256 * sizeof(uint64_t);
}

kvc_status kvc_residual_histograms(const kvc_layout* layout, const uint8_t* frames, int64_t n_chunks, uint64_t* d_hist,
                                   size_t hist_cap, void* stream) {
  ScoreParams p{};
  const kvc_status st = make_geo(layout, &p.g);
  if (st != KVC_OK) return st;
  if (n_chunks < 0 || n_chunks > (1 << 24)) return KVC_ERR_INVALID_ARG;
  if (n_chunks == 0) return KVC_OK;
  if (!frames || !d_hist || !aligned(frames, 8) || !aligned(d_hist, 8)) return KVC_ERR_INVALID_ARG;
  if (kvc_residual_histograms_size(layout, n_chunks) > hist_cap) return KVC_ERR_BUFFER_TOO_SMALL;
  p.frames = frames;
  p.n_chunks = (int32_t)n_chunks;
  p.hist = d_hist;
  return launch_residual_histograms(p, as_stream(stream));
}

double kvc_proxy_cost_bits(const kvc_layout* layout, const uint64_t* hist, int64_t n_chunks) {
  Geo g;
  if (make_geo(layout, &g) != KVC_OK || !hist || n_chunks < 0) return -1.0;
  const double pixels = (double)g.plane;
  double total = 0.0;
  for (int64_t s = 0; s < n_chunks * 2 * g.L; ++s) {
    double h[KVC_N_RESIDUALS];
    for (int k = 0; k < KVC_N_RESIDUALS; ++k) h[k] = histogram_entropy(hist + (s * KVC_N_RESIDUALS + k) * 256);
    total += pixels * (h[KVC_RES_LEFT] < h[KVC_RES_UP] ? h[KVC_RES_LEFT] : h[KVC_RES_UP]);
    if (g.F > 1) {
      double inter = h[KVC_RES_TIME];
      if (h[KVC_RES_TIME_LEFT] < inter) inter = h[KVC_RES_TIME_LEFT];
      if (h[KVC_RES_TIME_UP] < inter) inter = h[KVC_RES_TIME_UP];
      total += (double)(g.F - 1) * pixels * inter;
    }
  }
  return total;
}

int32_t kvc_tile_candidates(int32_t num_kv_heads, int32_t head_dim, int32_t* tile_h, int32_t* tile_w, int32_t* tile_seg,
                            int32_t cap) {
  if (num_kv_heads < 1 || head_dim < 1 || cap < 0 || (cap > 0 && (!tile_h || !tile_w || !tile_seg))) return -1;
  int32_t n = 0;
  for (int64_t h1 = 1; h1 <= num_kv_heads; h1 *= 2) {
    if (num_kv_heads % h1 != 0) continue;
    for (int64_t d1 = 1; d1 <= head_dim; d1 *= 2) {
      if (head_dim % d1 != 0 || head_dim / d1 < 8) continue;
      if (n < cap) {
        tile_h[n] = (int32_t)(h1 * d1);
        tile_w[n] = (int32_t)((num_kv_heads / h1) * (head_dim / d1));
        tile_seg[n] = (int32_t)(head_dim / d1);
      }
      ++n;
    }
  }
  return n;
}

kvc_status kvc_probe_expand(const void* d_src, void* d_dst, size_t out_bytes, const uint32_t* d_piece_map,
                            size_t piece_bytes, int32_t wg_bytes, int32_t shape, void* stream) {
  if (wg_bytes != 4096 && wg_bytes != 32768) return KVC_ERR_INVALID_ARG;
  if ((shape & ~(KVC_PROBE_ONE_XCD_PER_PIECE | KVC_PROBE_LINE_READS)) != 0) return KVC_ERR_INVALID_ARG;
  if (shape != 0 && (wg_bytes != 4096 || out_bytes % (8 * 4096) != 0)) return KVC_ERR_INVALID_ARG;
  if (piece_bytes < 32768 || (piece_bytes & (piece_bytes - 1)) != 0 || piece_bytes > ((size_t)1 << 30)) return KVC_ERR_INVALID_ARG;
  if (out_bytes % piece_bytes != 0 || out_bytes / piece_bytes > 0xffffffffull) return KVC_ERR_INVALID_ARG;
  if (out_bytes == 0) return KVC_OK;
  if (!d_src || !d_dst || !aligned(d_src, 8) || !aligned(d_dst, 16) || (d_piece_map && !aligned(d_piece_map, 4)))
    return KVC_ERR_INVALID_ARG;
  uint32_t log2_piece = 0;
  while (((size_t)1 << log2_piece) < piece_bytes) ++log2_piece;
  return launch_probe_expand(d_src, d_dst, out_bytes, d_piece_map, log2_piece, wg_bytes, shape, as_stream(stream));
}

size_t kvc_frame_size(const kvc_layout* layout) {
  Geo g;
  if (make_geo(layout, &g) != KVC_OK) return (size_t)-1;
  return (size_t)(3 * g.plane);
}

size_t kvc_frame_offset(const kvc_layout* layout, int32_t kind, int32_t layer_group, int32_t frame_index) {
  Geo g;
  if (make_geo(layout, &g) != KVC_OK) return (size_t)-1;
  if (kind < 0 || kind > 1 || layer_group < 0 || layer_group >= g.LG || frame_index < 0 || frame_index >= g.F)
    return (size_t)-1;
  return (size_t)((((int64_t)kind * g.LG + layer_group) * g.F + frame_index) * 3 * g.plane);
}

namespace {

// Fills the frame-call fields after fill_paged; first_token / n_tokens describe the chunk.
kvc_status fill_frames_args(RestoreParams& p, const uint8_t* frames, const void* meta, int64_t first_frame, int64_t n_frames,
                       int64_t n_tokens) {
  const int64_t per_chunk = (int64_t)2 * p.g.LG * p.g.F;
  if (first_frame < 0 || n_frames < 1 || first_frame >= per_chunk || n_frames > per_chunk - first_frame)
    return KVC_ERR_INVALID_ARG;
  if (n_tokens < 1 || n_tokens > p.g.T) return KVC_ERR_INVALID_ARG;
  if (!frames || !meta || !aligned(frames, 8) || !aligned(meta, 8)) return KVC_ERR_INVALID_ARG;  // 8-byte code loads
  p.frames = frames;
  p.meta = static_cast<const float*>(meta);
  p.frame_mode = 1;
  p.fm_first = (int32_t)first_frame;
  p.fm_count = p.fm_count1 = (int32_t)n_frames;
  p.fm_first2 = 0;
  p.frames2 = nullptr;
  return KVC_OK;
}

}  // namespace

kvc_status kvc_restore_paged_frames(const kvc_layout* layout, const uint8_t* frames, const void* meta, int64_t first_frame,
                                    int64_t n_frames, int64_t first_token, int64_t n_tokens, void* const* d_layer_cache,
                                    int64_t num_blocks, int32_t block_size, const int32_t* d_block_table,
                                    int64_t table_len, uint32_t* d_err, void* stream) {
  RestoreParams p{};
  kvc_status st = make_geo(layout, &p.g);
  if (st != KVC_OK) return st;
  if ((st = fill_paged(p, first_token, n_tokens, d_layer_cache, num_blocks, block_size, d_block_table, table_len,
                       d_err)) != KVC_OK)
    return st;
  if ((st = fill_frames_args(p, frames, meta, first_frame, n_frames, n_tokens)) != KVC_OK) return st;
  p.host_frames = in_host_memory(p.frames);
  return launch_restore(p, true, as_stream(stream));
}

kvc_status kvc_restore_paged_frame(const kvc_layout* layout, const uint8_t* frame, const void* meta, int32_t kind,
                                   int32_t layer_group, int32_t frame_index, int64_t first_token, int64_t n_tokens,
                                   void* const* d_layer_cache, int64_t num_blocks, int32_t block_size,
                                   const int32_t* d_block_table, int64_t table_len, uint32_t* d_err, void* stream) {
  Geo g;
  kvc_status st = make_geo(layout, &g);
  if (st != KVC_OK) return st;
  if (kind < 0 || kind > 1 || layer_group < 0 || layer_group >= g.LG || frame_index < 0 || frame_index >= g.F)
    return KVC_ERR_INVALID_ARG;
  return kvc_restore_paged_frames(layout, frame, meta, ((int64_t)kind * g.LG + layer_group) * g.F + frame_index, 1,
                                  first_token, n_tokens, d_layer_cache, num_blocks, block_size, d_block_table, table_len,
                                  d_err, stream);
}

namespace {

// {scale, mn} pairs of one layer of one chunk for a kind.
int64_t pairs_per_layer(const Geo& g, int kind) {
  return g.mode[kind] == KVC_Q_PER_CHANNEL ? (int64_t)g.C : (int64_t)g.T * g.H;
}

// HIP events of the fetch pipelines.  Creating and destroying events costs host time in front of every
// fetch, so the library keeps the events it has made, per device, for the life of the process: a call borrows
// what it needs and hands it back when it returns.  Handing back right after the work is enqueued is safe: a
// wait enqueued on a stream refers to the record that preceded it, not to later records of the same event, and
// an elapsed time is read before the call returns.
constexpr int kMaxDevices = 64;
std::mutex pool_mutex;
std::vector<hipEvent_t> pool_sync[kMaxDevices], pool_timed[kMaxDevices];

class EventLease {
 public:
  EventLease(int n_sync, int n_timed) {
    if (hipGetDevice(&device_) != hipSuccess || device_ < 0 || device_ >= kMaxDevices) {
      device_ = -1;
      return;
    }
    ok_ = take(pool_sync[device_], n_sync, hipEventDisableTiming, sync_) && take(pool_timed[device_], n_timed, hipEventDefault, timed_);
  }
  ~EventLease() {
    if (device_ < 0) return;
    std::lock_guard<std::mutex> lock(pool_mutex);
    pool_sync[device_].insert(pool_sync[device_].end(), sync_.begin(), sync_.end());
    pool_timed[device_].insert(pool_timed[device_].end(), timed_.begin(), timed_.end());
  }
  EventLease(const EventLease&) = delete;
  EventLease& operator=(const EventLease&) = delete;
  bool ok() const { return ok_; }
  hipEvent_t sync(int i) const { return sync_[i]; }
  hipEvent_t timed(int i) const { return timed_[i]; }

 private:
  static bool take(std::vector<hipEvent_t>& pool, int n, unsigned flags, std::vector<hipEvent_t>& out) {
    {
      std::lock_guard<std::mutex> lock(pool_mutex);
      while ((int)out.size() < n && !pool.empty()) {
        out.push_back(pool.back());
        pool.pop_back();
      }
    }
    while ((int)out.size() < n) {
      hipEvent_t e = nullptr;
      if (hipEventCreateWithFlags(&e, flags) != hipSuccess) return false;  // what was taken goes back in the destructor
      out.push_back(e);
    }
    return true;
  }
  int device_ = -1;
  bool ok_ = false;
  std::vector<hipEvent_t> sync_, timed_;
};

}  // namespace

size_t kvc_meta_staging_size(const kvc_layout* layout, int32_t order) {
  Geo g;
  if (make_geo(layout, &g) != KVC_OK) return (size_t)-1;
  if (order == KVC_ORDER_CHUNK) return (size_t)g.meta_floats * 4;
  if (order != KVC_ORDER_LAYER) return (size_t)-1;
  return (size_t)(3 * (pairs_per_layer(g, 0) + pairs_per_layer(g, 1)) * 8);
}

kvc_status kvc_fetch_pipeline_frames(const kvc_layout* layout, const kvc_host_chunk* chunks, int32_t n_chunks,
                                     void* const* d_frame_staging, size_t frame_staging_bytes, int32_t n_frame_staging,
                                     void* const* d_meta_staging, size_t meta_staging_bytes, int32_t n_meta_staging,
                                     void* const* d_layer_cache, int64_t num_blocks, int32_t block_size,
                                     const int32_t* d_block_table, int64_t table_len, uint32_t* d_err, void* copy_stream,
                                     void* compute_stream, int32_t order, void* const* group_ready_events,
                                     float* group_ready_ms, float* fetch_to_ready_ms) {
  RestoreParams base{};
  kvc_status st = make_geo(layout, &base.g);
  if (st != KVC_OK) return st;
  const Geo& g = base.g;
  if (order != KVC_ORDER_CHUNK && order != KVC_ORDER_LAYER) return KVC_ERR_INVALID_ARG;
  if (n_chunks < 0 || n_chunks > 4096) return KVC_ERR_INVALID_ARG;
  if (n_chunks == 0) {
    if (fetch_to_ready_ms) *fetch_to_ready_ms = 0.f;
    if (group_ready_ms)
      for (int lg = 0; lg < g.LG; ++lg) group_ready_ms[lg] = 0.f;
    return KVC_OK;
  }
  // n_frame_staging == 0: nothing is copied, the kernels read frames and pairs where they are
  const bool in_place = n_frame_staging == 0;
  if (!chunks || !compute_stream) return KVC_ERR_INVALID_ARG;
  if (!in_place) {
    if (!d_frame_staging || !d_meta_staging) return KVC_ERR_INVALID_ARG;
    if (n_frame_staging < 2 || n_frame_staging > 64 || n_meta_staging < 2 || n_meta_staging > 64) return KVC_ERR_INVALID_ARG;
    if (!copy_stream || copy_stream == compute_stream) return KVC_ERR_INVALID_ARG;
  }
  const size_t meta_off = kvc_blob_meta_offset(layout);
  const size_t meta_bytes = (size_t)g.meta_floats * 4, frame_size = (size_t)(3 * g.plane);
  const size_t blob_bytes = meta_off + meta_bytes;
  if (!in_place && (frame_staging_bytes < frame_size || meta_staging_bytes < kvc_meta_staging_size(layout, order)))
    return KVC_ERR_BUFFER_TOO_SMALL;
  int64_t total = 0;
  for (int i = 0; i < n_chunks; ++i) {
    if (!chunks[i].host_blob || (in_place && !aligned(chunks[i].host_blob, 8))) return KVC_ERR_INVALID_ARG;
    if (chunks[i].bytes < blob_bytes) return KVC_ERR_BUFFER_TOO_SMALL;
    if (chunks[i].n_tokens < 1 || chunks[i].n_tokens > g.T) return KVC_ERR_INVALID_ARG;
    if (i + 1 < n_chunks && chunks[i].n_tokens != g.T) return KVC_ERR_INVALID_ARG;
    total += chunks[i].n_tokens;
  }
  for (int s = 0; s < n_frame_staging; ++s)
    if (!d_frame_staging[s] || !aligned(d_frame_staging[s], 256)) return KVC_ERR_INVALID_ARG;
  for (int s = 0; s < n_meta_staging && !in_place; ++s)
    if (!d_meta_staging[s] || !aligned(d_meta_staging[s], 256)) return KVC_ERR_INVALID_ARG;
  if (group_ready_events)
    for (int lg = 0; lg < g.LG; ++lg)
      if (!group_ready_events[lg]) return KVC_ERR_INVALID_ARG;
  if ((st = fill_paged(base, 0, total, d_layer_cache, num_blocks, block_size, d_block_table, table_len, d_err)) != KVC_OK)
    return st;

  hipStream_t cs = as_stream(copy_stream), xs = as_stream(compute_stream);
  const bool blocking = fetch_to_ready_ms || group_ready_ms;
  if (in_place) {
    cs = xs;  // the only stream in use
    n_meta_staging = 0;
  }
  // "copied" after the copies into a frame slot, "freed" after the last kernel that read a slot (frame slots, then
  // meta slots); with timing: begin, end, then one per layer group
  EventLease ev(2 * n_frame_staging + n_meta_staging, blocking ? 2 + (group_ready_ms ? g.LG : 0) : 0);
  bool ok = ev.ok();
  const auto frames_copied = [&](int s) { return ev.sync(s); };
  const auto frames_freed = [&](int s) { return ev.sync(n_frame_staging + s); };
  const auto meta_freed = [&](int s) { return ev.sync(2 * n_frame_staging + s); };
  const hipEvent_t t_begin = ok && blocking ? ev.timed(0) : nullptr, t_end = ok && blocking ? ev.timed(1) : nullptr;
  const auto t_group = [&](int lg) { return ev.timed(2 + lg); };
  kvc_status result = ok ? KVC_OK : KVC_ERR_RUNTIME;

  // A slot of the frame ring is filled with pieces: runs of consecutive frames of one chunk,
  // copied back to back and announced with one event.  A piece reads the pairs of its meta
  // unit: the whole meta section of its chunk (chunk order) or the pairs of one layer group
  // of one chunk (layer order).
  struct Piece {
    int chunk;
    int64_t first, count;  // frames of the chunk
    size_t slot_off;       // bytes from the slot start
    int meta_slot;
    int lg;                // layer order: the group whose pairs the meta slot holds
    bool ends_unit;        // last piece that reads the meta slot's present content
  };
  const int64_t per_chunk = (int64_t)2 * g.LG * g.F;
  int64_t per_slot = (int64_t)(frame_staging_bytes / frame_size);
  if (per_slot > per_chunk) per_slot = per_chunk;
  std::vector<Piece> fill;       // pieces of the slot being filled
  int64_t fill_frames = 0;       // frames already in it
  int64_t fill_no = 0;           // slots filled so far
  int64_t fill_first_unit = 0;   // running number of the meta unit of the fill's first piece
  int64_t unit_no = -1;          // running number of the current meta unit

  auto flush = [&]() {
    if (fill.empty() || !ok) return;
    const int fs = (int)(fill_no % n_frame_staging);
    ok = hipEventRecord(frames_copied(fs), cs) == hipSuccess;  // covers the meta copies before it, too
    if (ok) ok = hipStreamWaitEvent(xs, frames_copied(fs), 0) == hipSuccess;
    for (size_t k = 0; k < fill.size() && ok; ++k) {
      const Piece& pc = fill[k];
      RestoreParams p = base;
      p.first_token = (int64_t)pc.chunk * g.T;
      p.n_tokens = chunks[pc.chunk].n_tokens;
      kvc_status ls = fill_frames_args(p, static_cast<const uint8_t*>(d_frame_staging[fs]) + pc.slot_off,
                                       d_meta_staging[pc.meta_slot], pc.first, pc.count, chunks[pc.chunk].n_tokens);
      if (order == KVC_ORDER_LAYER) {
        p.meta_sliced = 1;
        p.meta_l0 = 3 * pc.lg;
        p.moff[0] = 0;
        p.moff[1] = 3 * pairs_per_layer(g, 0) * 2;
      }
      if (ls == KVC_OK) ls = launch_restore(p, true, xs);
      if (ls != KVC_OK) {
        result = ls;
        ok = false;
        break;
      }
      if (pc.ends_unit) ok = hipEventRecord(meta_freed(pc.meta_slot), xs) == hipSuccess;
      // Layer group lg is complete once the last V frame of the last chunk has been restored
      // (everything else of the group is earlier in both orders).
      if (pc.chunk == n_chunks - 1)
        for (int lg = 0; lg < g.LG && ok; ++lg) {
          const int64_t last = ((int64_t)g.LG + lg) * g.F + g.F - 1;
          if (last < pc.first || last >= pc.first + pc.count) continue;
          if (group_ready_events) ok = hipEventRecord(static_cast<hipEvent_t>(group_ready_events[lg]), xs) == hipSuccess;
          if (ok && group_ready_ms) ok = hipEventRecord(t_group(lg), xs) == hipSuccess;
        }
    }
    if (ok) ok = hipEventRecord(frames_freed(fs), xs) == hipSuccess;
    fill.clear();
    fill_frames = 0;
    ++fill_no;
  };

  // Starts the meta unit of (chunk i, layer group lg or -1 for the whole section) and returns its slot.
  auto begin_unit = [&](int i, int lg) -> int {
    ++unit_no;
    // the slot about to be overwritten may still be needed by a piece of the unfinished fill
    if (!fill.empty() && fill_first_unit + n_meta_staging <= unit_no) flush();
    const int ms = (int)(unit_no % n_meta_staging);
    const uint8_t* src = static_cast<const uint8_t*>(chunks[i].host_blob) + meta_off;
    uint8_t* dst = static_cast<uint8_t*>(d_meta_staging[ms]);
    if (ok && unit_no >= n_meta_staging) ok = hipStreamWaitEvent(cs, meta_freed(ms), 0) == hipSuccess;
    if (lg < 0) {
      if (ok) ok = hipMemcpyAsync(dst, src, meta_bytes, hipMemcpyHostToDevice, cs) == hipSuccess;
    } else {
      const int nl = g.L - 3 * lg < 3 ? g.L - 3 * lg : 3;
      for (int kind = 0; kind < 2 && ok; ++kind) {
        const int64_t ppl = pairs_per_layer(g, kind);
        ok = hipMemcpyAsync(dst + (kind ? 3 * pairs_per_layer(g, 0) * 8 : 0),
                            src + (g.meta_off[kind] + 3 * lg * ppl * 2) * 4, (size_t)(nl * ppl * 8),
                            hipMemcpyHostToDevice, cs) == hipSuccess;
      }
    }
    return ms;
  };

  // Appends frames [first, first + count) of chunk i, cut into pieces that fit a slot.
  auto add_run = [&](int i, int64_t first, int64_t count, int ms, int lg, bool last_of_unit) {
    const uint8_t* blob = static_cast<const uint8_t*>(chunks[i].host_blob);
    while (count > 0 && ok) {
      if (fill_frames == per_slot) flush();
      const int64_t n = count < per_slot - fill_frames ? count : per_slot - fill_frames;
      const int fs = (int)(fill_no % n_frame_staging);
      if (fill.empty()) {
        fill_first_unit = unit_no;
        if (fill_no >= n_frame_staging) ok = hipStreamWaitEvent(cs, frames_freed(fs), 0) == hipSuccess;
      }
      const size_t off = (size_t)fill_frames * frame_size;
      if (ok)
        ok = hipMemcpyAsync(static_cast<uint8_t*>(d_frame_staging[fs]) + off, blob + (size_t)first * frame_size,
                            (size_t)n * frame_size, hipMemcpyHostToDevice, cs) == hipSuccess;
      fill.push_back(Piece{i, first, n, off, ms, lg, last_of_unit && n == count});
      fill_frames += n;
      first += n;
      count -= n;
    }
  };

  // K and V frames of one layer group of chunk i as one strided copy (two rows, LG * F frames apart in the
  // blob, back to back in the slot), when both runs still fit into the slot being filled.
  auto add_group_2d = [&](int i, int lg, int ms) -> bool {
    if (fill_frames == per_slot) flush();
    if (!ok || per_slot - fill_frames < 2 * (int64_t)g.F) return false;
    const uint8_t* blob = static_cast<const uint8_t*>(chunks[i].host_blob);
    const int fs = (int)(fill_no % n_frame_staging);
    if (fill.empty()) {
      fill_first_unit = unit_no;
      if (fill_no >= n_frame_staging) ok = hipStreamWaitEvent(cs, frames_freed(fs), 0) == hipSuccess;
    }
    const size_t off = (size_t)fill_frames * frame_size, run = (size_t)g.F * frame_size;
    if (ok)
      ok = hipMemcpy2DAsync(static_cast<uint8_t*>(d_frame_staging[fs]) + off, run, blob + (size_t)lg * run,
                            (size_t)g.LG * run, run, 2, hipMemcpyHostToDevice, cs) == hipSuccess;
    fill.push_back(Piece{i, (int64_t)lg * g.F, g.F, off, ms, lg, false});
    fill.push_back(Piece{i, ((int64_t)g.LG + lg) * g.F, g.F, off + run, ms, lg, true});
    fill_frames += 2 * (int64_t)g.F;
    return true;
  };

  // In place: one launch per run of consecutive frames, or per two runs of the same length (the K and the V
  // frames of a layer group, first2 > 0), reading the blob where it is.
  auto restore_in_place = [&](int i, int64_t first, int64_t count, int64_t first2) {
    if (!ok) return;
    const uint8_t* blob = static_cast<const uint8_t*>(chunks[i].host_blob);
    RestoreParams p = base;
    p.first_token = (int64_t)i * g.T;
    p.n_tokens = chunks[i].n_tokens;
    p.host_frames = 1;
    kvc_status ls = fill_frames_args(p, blob + (size_t)first * frame_size, blob + meta_off, first, count, chunks[i].n_tokens);
    if (ls == KVC_OK && first2 > 0) {
      p.fm_count = (int32_t)(2 * count);
      p.fm_first2 = (int32_t)first2;
      p.frames2 = blob + (size_t)first2 * frame_size;
    }
    if (ls == KVC_OK) ls = launch_restore(p, true, xs);
    if (ls != KVC_OK) {
      result = ls;
      ok = false;
    }
  };
  auto groups_ready = [&](int lg_first, int lg_end) {
    for (int lg = lg_first; lg < lg_end && ok; ++lg) {
      if (group_ready_events) ok = hipEventRecord(static_cast<hipEvent_t>(group_ready_events[lg]), xs) == hipSuccess;
      if (ok && group_ready_ms) ok = hipEventRecord(t_group(lg), xs) == hipSuccess;
    }
  };

  if (ok && in_place) {
    if (t_begin) ok = hipEventRecord(t_begin, xs) == hipSuccess;
    if (order == KVC_ORDER_CHUNK) {
      for (int i = 0; i < n_chunks; ++i) restore_in_place(i, 0, per_chunk, 0);
      groups_ready(0, g.LG);
    } else {
      for (int lg = 0; lg < g.LG && ok; ++lg) {
        for (int i = 0; i < n_chunks; ++i)  // K and V frames of the group
          restore_in_place(i, (int64_t)lg * g.F, g.F, ((int64_t)g.LG + lg) * g.F);
        groups_ready(lg, lg + 1);
      }
    }
  } else if (ok) {
    if (t_begin) ok = hipEventRecord(t_begin, cs) == hipSuccess;
    if (order == KVC_ORDER_CHUNK) {
      for (int i = 0; i < n_chunks && ok; ++i) {
        const int ms = begin_unit(i, -1);
        add_run(i, 0, per_chunk, ms, -1, true);
      }
    } else {
      // Appx A.3: the cache is filled layer by layer, so group 0 of every chunk comes first.
      for (int lg = 0; lg < g.LG && ok; ++lg)
        for (int i = 0; i < n_chunks && ok; ++i) {
          const int ms = begin_unit(i, lg);
          if (add_group_2d(i, lg, ms)) continue;
          add_run(i, (int64_t)lg * g.F, g.F, ms, lg, false);                   // K frames of the group
          add_run(i, ((int64_t)g.LG + lg) * g.F, g.F, ms, lg, true);           // V frames of the group
        }
    }
    flush();
  }
  if (ev.ok()) {
    if (!ok && result == KVC_OK) result = KVC_ERR_RUNTIME;
    if (blocking) {
      if (hipEventRecord(t_end, xs) != hipSuccess || hipEventSynchronize(t_end) != hipSuccess) {
        if (result == KVC_OK) result = KVC_ERR_RUNTIME;
      } else if (result == KVC_OK) {
        if (fetch_to_ready_ms && hipEventElapsedTime(fetch_to_ready_ms, t_begin, t_end) != hipSuccess)
          result = KVC_ERR_RUNTIME;
        if (group_ready_ms)
          for (int lg = 0; lg < g.LG && result == KVC_OK; ++lg)
            if (hipEventElapsedTime(&group_ready_ms[lg], t_begin, t_group(lg)) != hipSuccess) result = KVC_ERR_RUNTIME;
      }
    }
    if (result != KVC_OK) {
      (void)hipStreamSynchronize(cs);
      (void)hipStreamSynchronize(xs);
    }
  }
  return result;
}

namespace {

// Finite and not negative.  Tested on the bit pattern: this library is compiled with the
// assumption that no NaN occurs, so a floating-point comparison cannot be trusted to see one.
bool good_times(const double* t, int32_t n) {
  for (int32_t i = 0; i < n; ++i) {
    uint64_t b;
    memcpy(&b, &t[i], sizeof b);
    const bool negative = (b >> 63) != 0 && (b << 1) != 0;  // -0.0 counts as zero
    if (negative || ((b >> 52) & 0x7ffu) == 0x7ffu) return false;
  }
  return true;
}

}  // namespace

int32_t kvc_select_resolution(const double* size, const double* latency, const double* penalty, int32_t n_res,
                              int32_t n_loads, int32_t pool_load, int32_t active_res, double bandwidth,
                              double* bubble) {
  if (!size || !latency || !penalty || n_res < 1 || n_loads < 1 || n_res > (1 << 20) || n_loads > (1 << 20)) return -1;
  if (pool_load < 1 || pool_load > n_loads || active_res < -1 || active_res >= n_res) return -1;
  if (!good_times(&bandwidth, 1) || bandwidth == 0.0) return -1;
  const double* row = latency + (size_t)(pool_load - 1) * n_res;
  if (!good_times(size, n_res) || !good_times(penalty, n_res) || !good_times(row, n_res)) return -1;
  // idle gap of version r: when it has arrived against when the pool is ready for it
  const auto gap = [&](int32_t r) {
    const double switch_cost = (active_res >= 0 && r != active_res) ? penalty[r] : 0.0;
    const double d = size[r] / bandwidth - row[r] - switch_cost;  // subtracted in this order (left to right)
    return d < 0.0 ? -d : d;
  };
  const int32_t best = first_argmin(n_res, gap);
  if (bubble) *bubble = gap(best);
  return best;
}

double kvc_est_bandwidth(double last_chunk_size, double last_transmission_delay) {
  if (!good_times(&last_chunk_size, 1) || !good_times(&last_transmission_delay, 1)) return -1.0;
  if (last_chunk_size == 0.0 || last_transmission_delay == 0.0) return -1.0;
  return last_chunk_size / last_transmission_delay;
}

kvc_status kvc_layout_set_resolution(kvc_layout* layout, int32_t width, int32_t height) {
  if (!layout || width < 1 || height < 1) return KVC_ERR_INVALID_ARG;
  if (layout->tile_w < 1 || layout->tile_h < 1) return KVC_ERR_INVALID_ARG;
  const int32_t tx = width / layout->tile_w, ty = height / layout->tile_h;
  layout->tiles_x = tx < 1 ? 1 : tx;
  layout->tiles_y = ty < 1 ? 1 : ty;
  return kvc_layout_validate(layout);
}

int32_t kvc_admission_min_buffered(const double* t_fetch, const double* t_comp, int32_t n_stages) {
  if (!t_fetch || !t_comp || n_stages < 1 || !good_times(t_fetch, n_stages) || !good_times(t_comp, n_stages)) return -1;
  // The condition for k does not depend on n_buffered, so the answer is the largest k that violates it.
  double fetched = 0.0, computed = 0.0;  // sum_{j<=k} t_fetch, sum_{j<=k-1} t_comp
  int32_t need = 0;
  for (int32_t k = 1; k <= n_stages; ++k) {
    fetched += t_fetch[k - 1];
    if (k >= 2) computed += t_comp[k - 2];
    if (fetched > computed) need = k;
  }
  return need;
}

int32_t kvc_admission_ok(const double* t_fetch, const double* t_comp, int32_t n_stages, int32_t n_buffered) {
  if (n_buffered < 0 || n_buffered > n_stages) return -1;
  const int32_t need = kvc_admission_min_buffered(t_fetch, t_comp, n_stages);
  if (need < 0) return -1;
  return n_buffered >= need ? 1 : 0;
}

kvc_status kvc_fetch_pipeline(const kvc_layout* layout, const kvc_host_chunk* chunks, int32_t n_chunks,
                              void* const* d_staging, size_t staging_bytes, int32_t n_staging,
                              void* const* d_layer_cache, int64_t num_blocks, int32_t block_size,
                              const int32_t* d_block_table, int64_t table_len, uint32_t* d_err, void* copy_stream,
                              void* compute_stream, float* fetch_to_ready_ms) {
  RestoreParams base{};
  kvc_status st = make_geo(layout, &base.g);
  if (st != KVC_OK) return st;
  if (n_chunks < 0 || n_chunks > 4096) return KVC_ERR_INVALID_ARG;
  if (n_chunks == 0) {
    if (fetch_to_ready_ms) *fetch_to_ready_ms = 0.f;
    return KVC_OK;
  }
  // n_staging == 0: no copies at all, the restore kernels read the blobs where they are
  const bool in_place = n_staging == 0;
  if (!chunks || !compute_stream) return KVC_ERR_INVALID_ARG;
  if (!in_place) {
    if (!d_staging || n_staging < 2 || n_staging > 64) return KVC_ERR_INVALID_ARG;
    if (!copy_stream || copy_stream == compute_stream) return KVC_ERR_INVALID_ARG;
  }
  const size_t meta_off = kvc_blob_meta_offset(layout);
  const size_t blob_bytes = meta_off + (size_t)base.g.meta_floats * 4;
  if (!in_place && staging_bytes < blob_bytes) return KVC_ERR_BUFFER_TOO_SMALL;
  int64_t total = 0;
  for (int i = 0; i < n_chunks; ++i) {
    if (!chunks[i].host_blob || (in_place && !aligned(chunks[i].host_blob, 8))) return KVC_ERR_INVALID_ARG;
    if (chunks[i].bytes < blob_bytes) return KVC_ERR_BUFFER_TOO_SMALL;
    if (chunks[i].n_tokens < 1 || chunks[i].n_tokens > base.g.T) return KVC_ERR_INVALID_ARG;
    if (i + 1 < n_chunks && chunks[i].n_tokens != base.g.T) return KVC_ERR_INVALID_ARG;
    total += chunks[i].n_tokens;
  }
  for (int s = 0; s < n_staging; ++s)
    if (!d_staging[s] || !aligned(d_staging[s], 256)) return KVC_ERR_INVALID_ARG;
  // whole-range check of the paged destination before anything is enqueued
  if ((st = fill_paged(base, 0, total, d_layer_cache, num_blocks, block_size, d_block_table, table_len, d_err)) != KVC_OK)
    return st;

  hipStream_t cs = as_stream(copy_stream), xs = as_stream(compute_stream);
  // Per staging slot: "copied" after the copy into it, "slot free" after the restore that read it.
  if (in_place) cs = xs;  // the only stream in use
  EventLease ev(2 * n_staging, fetch_to_ready_ms ? 2 : 0);
  bool ok = ev.ok();
  const auto copied = [&](int slot) { return ev.sync(slot); };
  const auto freed = [&](int slot) { return ev.sync(n_staging + slot); };
  const hipEvent_t t_begin = ok && fetch_to_ready_ms ? ev.timed(0) : nullptr;
  const hipEvent_t t_end = ok && fetch_to_ready_ms ? ev.timed(1) : nullptr;
  kvc_status result = ok ? KVC_OK : KVC_ERR_RUNTIME;

  if (ok) {
    if (t_begin) ok = hipEventRecord(t_begin, cs) == hipSuccess;
    for (int i = 0; i < n_chunks && ok; ++i) {
      const int s = in_place ? 0 : i % n_staging;
      const void* blob = chunks[i].host_blob;
      if (!in_place) {
        // the copy into slot s must wait for the restore that last read it
        if (i >= n_staging) ok = hipStreamWaitEvent(cs, freed(s), 0) == hipSuccess;
        if (ok) ok = hipMemcpyAsync(d_staging[s], chunks[i].host_blob, blob_bytes, hipMemcpyHostToDevice, cs) == hipSuccess;
        if (ok) ok = hipEventRecord(copied(s), cs) == hipSuccess;
        if (ok) ok = hipStreamWaitEvent(xs, copied(s), 0) == hipSuccess;
        if (!ok) break;
        blob = d_staging[s];
      }
      RestoreParams p = base;
      p.host_frames = in_place;
      p.frames = static_cast<const uint8_t*>(blob);
      p.meta = reinterpret_cast<const float*>(static_cast<const uint8_t*>(blob) + meta_off);
      p.first_token = (int64_t)i * base.g.T;
      p.n_tokens = chunks[i].n_tokens;
      const kvc_status ls = launch_restore(p, true, xs);
      if (ls != KVC_OK) {
        result = ls;
        ok = false;
        break;
      }
      if (!in_place) ok = hipEventRecord(freed(s), xs) == hipSuccess;
    }
    if (!ok && result == KVC_OK) result = KVC_ERR_RUNTIME;
    if (t_end) {
      // compute_stream is the later of the two by construction
      if (hipEventRecord(t_end, xs) != hipSuccess || hipEventSynchronize(t_end) != hipSuccess) {
        if (result == KVC_OK) result = KVC_ERR_RUNTIME;
      } else if (result == KVC_OK) {
        // t_begin sits on the copy stream, t_end on the compute stream
        if (hipEventElapsedTime(fetch_to_ready_ms, t_begin, t_end) != hipSuccess) result = KVC_ERR_RUNTIME;
      }
    } else if (result != KVC_OK) {
      // part of the work may be queued: let it drain before the events go away
      (void)hipStreamSynchronize(cs);
      (void)hipStreamSynchronize(xs);
    }
  }
  return result;
}

}  // extern "C"
