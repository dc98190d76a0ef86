/*
 * kvc.h -- C ABI of libkvc: the pack / restore hot path of video-codec based
 * remote KV-cache reuse (KVCodec, arXiv 2602.09725) on one AMD MI355X (gfx950).
 *
 * What the library computes
 * -------------------------
 * Compress side (Sec. 3.2 "Codec-friendly KV Compression", Sec. 4 item (1)):
 * the KV cache of an inference engine, shape [token, layer, head_num, head_dim]
 * (Sec. 3.2, first paragraph), is quantized to 8-bit integers and laid out as
 * video frames [frame, height, width, 3]:
 *   - inter-frame layout (Sec. 3.2.1, steps 1-3): three consecutive layers
 *     become the three colour planes of a frame; the T token tensors of a chunk
 *     are split into groups of F adjacent tokens, and the F tensors of a group
 *     occupy the same tile position in F consecutive frames;
 *   - intra-frame layout (Sec. 3.2.2, rules i-iii and the tiles (8,512),
 *     (8,128), (16,64) found there): the head_num*head_dim vector of one token
 *     and layer is re-tiled into a (tile_h, tile_w) block with no permutation of
 *     heads or of elements inside a head: row-major, or as the two-level
 *     reshape head_num -> (h1, h2), head_dim -> (d1, d2), tile (h1*d1, h2*d2)
 *     of the section's (32,128) -> (8,4) x (1,128) -> (8,512) example.
 * Fetch side (Sec. 3.3.2 "Frame-wise KV tensor restoration", Sec. 4 item (2)):
 * decoded frames are mapped back to KV tensors, dequantized and written into the
 * preallocated slots of the engine's paged memory.  The H.265 encoder / decoder
 * between the two sides is lossless (Sec. 4 item (1)), so frames out == frames
 * in, and it is not part of this library: frames are an opaque byte boundary.
 * The pipelined fetcher follows the transmission/decoding overlap of Sec. 3.3.2
 * ("Adaptive resolution KV fetching", first paragraph) with host->device copies
 * of frame buffers standing in for the transmission stage.
 *
 * Notation: L layers, H KV heads, D head_dim, C = H*D, T = chunk_tokens,
 * (th, tw) = tile with th*tw == C, (TX, TY) = tile grid of a frame,
 * G = TX*TY tile positions, F = ceil(T / G) frames per layer group,
 * LG = ceil(L / 3) layer groups, W = TX*tw, Hp = TY*th.
 *
 * Quantizer (Sec. 4 item (1) states only that the tensors become integers
 * before encoding; the 8-bit asymmetric affine form is this library's definition), all in fp32:
 *   group  : KVC_Q_PER_CHANNEL -> one (chunk, kind, layer, head, dim) over the
 *            chunk's valid tokens; KVC_Q_PER_TOKEN -> one (kind, layer, token,
 *            head) over the D elements of the head
 *   mn     = min + 0.0f (so -0.0 becomes +0.0), range = max - mn
 *   scale  = range / 255, inv = 255 / range (both correctly rounded; 0 if range==0)
 *   code   = clamp(rint((x - mn) * inv), 0, 255)   rint = round half to even
 *   x_hat  = fma(code, scale, mn), rounded to nearest even into fp16 / bf16
 *
 * Byte layouts
 * ------------
 * frames : [chunk][kind(K=0,V=1)][LG][F][3][Hp][W] uint8, planar.  The byte of
 *          element (kind, l, t, h, d), t local to the chunk, sits at
 *            e = h*D + d ; r = e / tw ; cc = e % tw            (tile_seg == 0)
 *            r = (h / h2)*d1 + d / d2 ; cc = (h % h2)*d2 + d % d2,
 *              d2 = tile_seg, d1 = D / d2, h2 = tw / d2        (tile_seg  > 0)
 *            f = t % F   ; g = t / F  ; ty = g / TX ; tx = g % TX
 *            y = ty*th + r ; x = tx*tw + cc ; lg = l / 3 ; pl = l % 3
 *          Every byte no valid element maps to (planes of layers >= L, tiles of
 *          tokens beyond the chunk's valid count) is 0.
 * meta   : per chunk [K block][V block] of {scale, mn} fp32 pairs;
 *          per-channel block = [L][H][D] pairs, per-token block = [L][T][H]
 *          pairs (pairs of tokens beyond the valid count are {0, 0}).
 * Multi-chunk buffers are arrays of fixed-stride chunk sections:
 * frames = n_chunks * frame_bytes, meta = n_chunks * meta_bytes, with
 * n_chunks = ceil(n_tokens / T); only the last chunk may be short.
 * blob   : one chunk as shipped to a fetcher: its frame section, zero padding up
 *          to kvc_blob_meta_offset() (frame_bytes rounded up to 256), then its
 *          meta section.
 *
 * Conventions
 * -----------
 * Pointers marked DEVICE must be device memory valid on the current HIP device;
 * pointers marked HOST are ordinary host memory (PINNED where stated).  The
 * caller owns every buffer; the library allocates no device memory and keeps no
 * reference to a caller's buffer after a call returns.  Its only state is a
 * per-device pool of HIP events that the two fetch pipelines borrow from: the
 * events are created on first use, reused by later calls and released when the
 * process ends.  Data calls enqueue work on the given stream
 * (a hipStream_t passed as void*, NULL = the default stream) and return without
 * synchronizing unless stated.  Every host-checkable fault returns an error
 * code before anything is enqueued; nothing throws across the ABI.  Calls are
 * thread-safe for distinct streams.  Inputs must be finite; for each group
 * either max == min or (max - min) >= 2^-100.
 * Required alignment: kv / cache base pointers and strides 16 bytes, frames
 * 16 bytes, meta 8 bytes; otherwise KVC_ERR_INVALID_ARG.
 */
#ifndef KVC_H
#define KVC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define KVC_ABI_VERSION 2u

typedef enum {
  KVC_OK = 0,
  KVC_ERR_INVALID_ARG = 1,      /* null pointer, inconsistent layout, bad alignment, bad range */
  KVC_ERR_UNSUPPORTED = 2,      /* well-formed request outside what the kernels cover        */
  KVC_ERR_BUFFER_TOO_SMALL = 3, /* a capacity argument is smaller than the call needs         */
  KVC_ERR_RUNTIME = 4           /* a HIP runtime call failed                                   */
} kvc_status;

typedef enum { KVC_F16 = 0, KVC_BF16 = 1 } kvc_dtype;
typedef enum { KVC_Q_PER_CHANNEL = 0, KVC_Q_PER_TOKEN = 1 } kvc_qmode;

/* Geometry of one packed stream.  Read on the host during a call only. */
typedef struct {
  uint32_t struct_size;  /* sizeof(kvc_layout) as the caller compiled it           */
  uint32_t abi_version;  /* KVC_ABI_VERSION                                        */
  int32_t num_layers;    /* L >= 1                                                 */
  int32_t num_kv_heads;  /* H >= 1                                                 */
  int32_t head_dim;      /* D >= 1; a multiple of 8, else KVC_ERR_UNSUPPORTED      */
  int32_t dtype;         /* kvc_dtype of the KV tensors                            */
  int32_t chunk_tokens;  /* T >= 1 tokens per chunk (Sec. 4 item (1): chunking)    */
  int32_t tile_h;        /* th, tile_h*tile_w == H*D (Sec. 3.2.2)                  */
  int32_t tile_w;        /* tw; a multiple of 8, else KVC_ERR_UNSUPPORTED          */
  int32_t tiles_x;       /* TX: tiles per frame row; sets the frame resolution     */
  int32_t tiles_y;       /* TY: tiles per frame column (Sec. 3.2.1 observation iii)*/
  int32_t k_mode;        /* kvc_qmode for K (default per channel)                  */
  int32_t v_mode;        /* kvc_qmode for V (default per token)                    */
  int32_t tile_seg;      /* 0: the tile is the row-major reshape of the H*D vector.
                            d2 > 0: two-level tiling of Sec. 3.2.2 -- head_num
                            reshaped to (h1, h2), head_dim to (d1, d2), tile =
                            (h1*d1, h2*d2); d2 divides D and tile_w, tile_w/d2
                            divides H; a multiple of 8, else KVC_ERR_UNSUPPORTED */
} kvc_layout;

/* Strides of a contiguous-style KV tensor [L][2][tokens][H][D], in ELEMENTS.
 * The innermost [H][D] block of one token is contiguous.  Each stride must be a
 * multiple of 8 elements. */
typedef struct {
  int64_t layer_stride;
  int64_t kv_stride;
  int64_t token_stride;
} kvc_strides;

/* One chunk blob in PINNED HOST memory (see "blob" above). */
typedef struct {
  const void* host_blob;
  size_t bytes;     /* >= kvc_blob_meta_offset + meta_bytes */
  int64_t n_tokens; /* valid tokens of this chunk, 1..T      */
} kvc_host_chunk;

/* Checks a layout for internal consistency (sizes positive, tile product,
 * struct_size / abi_version).  HOST pointer. */
kvc_status kvc_layout_validate(const kvc_layout* layout);

/* Sizes of one chunk section.  Any output pointer may be NULL.
 * frame_bytes = 2*LG*F*3*Hp*W ; meta_bytes = 8 * (pairs of K block + V block);
 * frames_per_group = F (Sec. 3.2.1 step 2). */
kvc_status kvc_chunk_sizes(const kvc_layout* layout, size_t* frame_bytes, size_t* meta_bytes,
                           int32_t* frames_per_group);

/* Offset of the meta section inside a chunk blob; blob size = offset + meta_bytes. */
size_t kvc_blob_meta_offset(const kvc_layout* layout);

/* Compress side: quantize + codec-friendly layout (Sec. 3.2.1 steps 1-3,
 * Sec. 3.2.2, Sec. 4 item (1)).
 *   kv        DEVICE in : [L][2][n_tokens][H][D] fp16|bf16 addressed by `strides`
 *   n_tokens  tokens to pack (0 is allowed and does nothing)
 *   frames    DEVICE out: ceil(n_tokens/T) chunk sections, every byte written
 *   meta      DEVICE out: ceil(n_tokens/T) chunk sections, every byte written
 *   *_cap     capacities in bytes; too small -> KVC_ERR_BUFFER_TOO_SMALL */
kvc_status kvc_pack(const kvc_layout* layout, const void* kv, kvc_strides strides, int64_t n_tokens,
                    uint8_t* frames, size_t frames_cap, void* meta, size_t meta_cap, void* stream);

/* How kvc_pack would run for this layout and these strides: host arithmetic
 * only, nothing is enqueued (Sec. 4 item (1), the offline compression pass).
 *   *resident  HOST out, nullable: 1 when the strip of channels a workgroup
 *              quantizes per channel is held in registers for a whole chunk, so
 *              the input is read from memory once; 0 when only the last 3072
 *              tokens of a chunk's strip wait on chip and the tokens before them
 *              are read twice (chunk_tokens > 2048, or 2048 * token_stride * 2
 *              bytes does not fit the 32-bit offsets of the register-resident
 *              body), or when no kind is quantized per channel
 *   *threads   HOST out, nullable: threads per workgroup of the launch
 * Returns the status kvc_pack would return for the same layout and strides. */
kvc_status kvc_pack_plan(const kvc_layout* layout, kvc_strides strides, int32_t* resident, int32_t* threads);

/* Fetch side into a contiguous tensor (Sec. 3.3.2 frame-wise restoration:
 * unpack + dequantize).
 *   frames, meta  DEVICE in : chunk sections as written by kvc_pack
 *   kv_out        DEVICE out: [L][2][n_tokens][H][D] addressed by `strides`;
 *                 only the n_tokens valid tokens are written. */
kvc_status kvc_restore(const kvc_layout* layout, const uint8_t* frames, const void* meta,
                       int64_t n_tokens, void* kv_out, kvc_strides strides, void* stream);

/* Fetch side into the engine's paged memory (Sec. 3.3.2: restored tensors go
 * straight to slots the engine has already allocated in its paged memory;
 * Sec. 4 item (2): the sparse frame-to-paged-memory transfer operator).
 *   frames, meta   DEVICE in : sections of the chunks that hold sequence
 *                  positions [first_token, first_token + n_tokens).  Either
 *                  may also be pinned host memory that is mapped into the
 *                  device (hipHostMalloc): the kernel then reads it over the
 *                  host link and no staging copy is needed.
 *   first_token    absolute position of token 0 of `frames`; multiple of T
 *   d_layer_cache  DEVICE in : array of L DEVICE pointers, layer l's cache is
 *                  [2][num_blocks][block_size][H][D] of the layout's dtype
 *   d_block_table  DEVICE in : int32[table_len], logical block -> physical
 *                  block; token p goes to block d_block_table[p / block_size],
 *                  slot p % block_size; needs
 *                  table_len*block_size >= first_token + n_tokens
 *   d_err          DEVICE in/out, may be NULL: a physical id outside
 *                  [0, num_blocks) cannot be seen from the host; the kernel
 *                  skips the writes of that block and ORs 1 into *d_err. */
kvc_status kvc_restore_paged(const kvc_layout* layout, const uint8_t* frames, const void* meta,
                             int64_t first_token, int64_t n_tokens, void* const* d_layer_cache,
                             int64_t num_blocks, int32_t block_size, const int32_t* d_block_table,
                             int64_t table_len, uint32_t* d_err, void* stream);

/* Pipelined fetcher (Sec. 3.3.2: transmission overlapped with decoding, the
 * restoration riding along; the compressed data waits in a host-memory buffer).
 * Chunk i (holding sequence positions i*T ...) is copied from its pinned HOST
 * blob to staging slot i % n_staging on `copy_stream`, then restored into the
 * paged cache on `compute_stream`; a slot is reused only after the restore that
 * read it has finished.  Every chunk but the last must hold T tokens.
 *   chunks            HOST array of n_chunks descriptors (blobs PINNED HOST)
 *   d_staging         HOST array of n_staging DEVICE buffers, each >= blob size
 *   staging_bytes     capacity of each staging buffer
 *   n_staging         2..64, or 0: nothing is copied, the restore kernels read
 *                     the blobs in place over the host link (the blobs must then
 *                     be mapped into the device, as hipHostMalloc memory is, and
 *                     8-byte aligned; d_staging, staging_bytes and copy_stream
 *                     are not looked at).  With tiles narrower than 512 bytes in
 *                     rows of tiles of at least 512 the kernel's reads are long
 *                     enough to draw the link's full rate, and this form is the
 *                     faster one
 *   copy_stream, compute_stream : two distinct non-NULL hipStream_t
 *   fetch_to_ready_ms HOST out, may be NULL.  If non-NULL the call blocks until
 *                     the last restore has finished and stores the time from
 *                     the first copy being enqueued to that moment; if NULL the
 *                     call returns after enqueueing and the caller synchronizes
 *                     compute_stream. */
kvc_status kvc_fetch_pipeline(const kvc_layout* layout, const kvc_host_chunk* chunks, int32_t n_chunks,
                              void* const* d_staging, size_t staging_bytes, int32_t n_staging,
                              void* const* d_layer_cache, int64_t num_blocks, int32_t block_size,
                              const int32_t* d_block_table, int64_t table_len, uint32_t* d_err,
                              void* copy_stream, void* compute_stream, float* fetch_to_ready_ms);

/* Frame-wise restoration (Sec. 3.3.2: a frame is mapped back to KV tensors and
 * placed into the preallocated paged slots as soon as it is available, so the
 * decompress buffer holds frames, not chunks).
 * Frames of a chunk are numbered in storage order,
 *   frame number = (kind * LG + layer_group) * F + frame_index;
 * one frame = the three planes [3][Hp][W] and carries, for the layers
 * 3*layer_group .. +2 that exist, the tokens t of the chunk with
 * t % F == frame_index (Sec. 3.2.1 step 3).
 *   frames       DEVICE in : n_frames consecutive frames, n_frames*3*Hp*W bytes,
 *                as they sit in the chunk section from byte
 *                first_frame * kvc_frame_size(layout) on; 8-byte aligned
 *   meta         DEVICE in : the meta section of the chunk the frames belong to
 *                (either may be pinned host memory mapped into the device, as
 *                for kvc_restore_paged)
 *   first_frame, n_frames : 0 <= first_frame, n_frames >= 1,
 *                first_frame + n_frames <= 2*LG*F
 *   first_token  absolute position of the chunk's token 0 (multiple of T)
 *   n_tokens     valid tokens of that chunk, 1..T
 * Destination and error behaviour as kvc_restore_paged.  Restoring every frame of
 * a chunk, in any order and any grouping, gives the same cache as one
 * kvc_restore_paged call on the chunk. */
kvc_status kvc_restore_paged_frames(const kvc_layout* layout, const uint8_t* frames, const void* meta,
                                    int64_t first_frame, int64_t n_frames, int64_t first_token, int64_t n_tokens,
                                    void* const* d_layer_cache, int64_t num_blocks, int32_t block_size,
                                    const int32_t* d_block_table, int64_t table_len, uint32_t* d_err, void* stream);

/* The same for the single frame (kind, layer_group, frame_index). */
kvc_status kvc_restore_paged_frame(const kvc_layout* layout, const uint8_t* frame, const void* meta, int32_t kind,
                                   int32_t layer_group, int32_t frame_index, int64_t first_token, int64_t n_tokens,
                                   void* const* d_layer_cache, int64_t num_blocks, int32_t block_size,
                                   const int32_t* d_block_table, int64_t table_len, uint32_t* d_err, void* stream);

/* Bytes of one frame (3*Hp*W) and the offset of frame (kind, layer_group,
 * frame_index) inside a chunk's frame section; (size_t)-1 on a bad argument. */
size_t kvc_frame_size(const kvc_layout* layout);
size_t kvc_frame_offset(const kvc_layout* layout, int32_t kind, int32_t layer_group, int32_t frame_index);

/* Order in which kvc_fetch_pipeline_frames moves the frames of a request. */
typedef enum kvc_fetch_order {
  KVC_ORDER_CHUNK = 0, /* chunk by chunk, each chunk in storage order                  */
  KVC_ORDER_LAYER = 1  /* layer group by layer group (Appx A.3: the preallocated cache
                          is filled layer by layer so that inference can start on the
                          first layers while later ones are still being fetched); inside
                          a group chunk by chunk, K frames then V frames                 */
} kvc_fetch_order;

/* Bytes one meta staging buffer of kvc_fetch_pipeline_frames must hold: a whole
 * chunk meta section (KVC_ORDER_CHUNK) or the pairs of the three layers of one
 * layer group of one chunk (KVC_ORDER_LAYER).  (size_t)-1 on a bad argument. */
size_t kvc_meta_staging_size(const kvc_layout* layout, int32_t order);

/* Pipelined fetcher at frame granularity: as kvc_fetch_pipeline, but the device
 * staging holds a few frames and a few meta pieces instead of whole chunk
 * blobs -- the frame-wise decompress buffer of Sec. 3.3.2 -- and the order of the
 * frames is selectable.  Runs of consecutive frames are copied into a frame
 * staging buffer until it is full (it holds floor(frame_staging_bytes /
 * kvc_frame_size) frames, at most a chunk's), announced with one event and
 * restored with one kvc_restore_paged_frames launch per run; the pairs a run
 * needs are copied before it.  In KVC_ORDER_LAYER a buffer that holds at least
 * 2*F frames receives the K and the V frames of a (chunk, layer group) in one
 * two-row strided copy.
 *   d_frame_staging  HOST array of n_frame_staging (2..64) DEVICE buffers of
 *                    frame_staging_bytes >= kvc_frame_size, 256-byte aligned.
 *                    n_frame_staging = 0: nothing is copied; every run of
 *                    frames (a whole chunk in KVC_ORDER_CHUNK, the K and the V
 *                    frames of a (chunk, layer group) in KVC_ORDER_LAYER) is
 *                    restored by a kernel that reads the blob in place over the
 *                    host link, on compute_stream alone (blobs mapped into the
 *                    device and 8-byte aligned; both staging arrays, their sizes
 *                    and copy_stream are not looked at)
 *   d_meta_staging   HOST array of n_meta_staging (2..64) DEVICE buffers of
 *                    meta_staging_bytes >= kvc_meta_staging_size(layout, order),
 *                    256-byte aligned
 *   order            a kvc_fetch_order
 *   group_ready_events  HOST array of LG hipEvent_t created by the caller, or
 *                    NULL.  Event g is recorded on compute_stream once every
 *                    token of layers 3g .. 3g+2 (K and V, all chunks) is in the
 *                    cache: the per-layer state an engine needs for the
 *                    non-blocking condition of Appx A.3 (kvc_admission_*).
 *   group_ready_ms   HOST out float[LG] or NULL: time from the first copy being
 *                    enqueued to each group being ready.
 *   fetch_to_ready_ms HOST out or NULL.  The call blocks until the last restore
 *                    has finished if either time output is non-NULL; otherwise it
 *                    returns after enqueueing.  In that form it enqueues copies,
 *                    kernels and event edges only, so it may be recorded into a
 *                    HIP graph by stream capture (begin the capture on
 *                    copy_stream and make it wait for compute_stream before the
 *                    capture ends) and replayed.
 * Other arguments, blob format and error behaviour as kvc_fetch_pipeline. */
kvc_status kvc_fetch_pipeline_frames(const kvc_layout* layout, const kvc_host_chunk* chunks, int32_t n_chunks,
                                     void* const* d_frame_staging, size_t frame_staging_bytes, int32_t n_frame_staging,
                                     void* const* d_meta_staging, size_t meta_staging_bytes, int32_t n_meta_staging,
                                     void* const* d_layer_cache, int64_t num_blocks, int32_t block_size,
                                     const int32_t* d_block_table, int64_t table_len, uint32_t* d_err, void* copy_stream,
                                     void* compute_stream, int32_t order, void* const* group_ready_events,
                                     float* group_ready_ms, float* fetch_to_ready_ms);

/* Non-blocking condition of the layer-wise fetching-inference pipeline (Appx
 * A.3), host arithmetic only.  Stage j (1-based in the paper, index j-1 here) is
 * a layer or a layer group; t_fetch[j-1] is the time to make its KV ready (the
 * paper's per-layer decoding time), t_comp[j-1] its inference time.  With
 * n_buffered stages already in the cache the request may join the running
 * queue iff for every k in n_buffered+1 .. n_stages
 *     sum_{j=1..k} t_fetch[j] <= sum_{j=1..k-1} t_comp[j].
 * kvc_admission_ok returns 1 if the condition holds, 0 if not, -1 on a bad
 * argument (NULL, n_stages < 1, n_buffered outside 0..n_stages, a negative or
 * non-finite time).  kvc_admission_min_buffered returns the smallest n_buffered
 * for which it holds (n_stages if every stage must be buffered first), -1 on a
 * bad argument.  Sums are accumulated in double in index order. */
int32_t kvc_admission_ok(const double* t_fetch, const double* t_comp, int32_t n_stages, int32_t n_buffered);
int32_t kvc_admission_min_buffered(const double* t_fetch, const double* t_comp, int32_t n_stages);

/* Adaptive-resolution selector (Alg. 1, Appx A.2; Sec. 3.3.1), host arithmetic
 * only.  A chunk version is a good fit for the network and the decode pool when
 * it arrives just as the pool has finished the work in front of it.  For
 * version r the two times are
 *   arrival[r] = size[r] / bandwidth
 *   ready[r]   = latency[(pool_load - 1) * n_res + r]   (profile table: one row
 *                per pool load) + penalty[r] when the pool has to switch, i.e.
 *                active_res >= 0 and r != active_res
 * and the call returns the r that minimizes the idle gap |arrival[r] - ready[r]|
 * (the lowest index among equal gaps); *bubble (may be NULL) gets that gap.
 * size and bandwidth share a unit (bytes and bytes/s, MB and MB/s, ...).
 *   pool_load   present load of the decode pool, 1..n_loads
 *   active_res  resolution the pool is working on, or -1 for an idle pool
 * Returns -1 on a bad argument (NULL, n_res < 1, n_loads < 1, pool_load or
 * active_res out of range, bandwidth not finite or <= 0, a negative or
 * non-finite table entry). */
int32_t kvc_select_resolution(const double* size, const double* latency, const double* penalty, int32_t n_res,
                              int32_t n_loads, int32_t pool_load, int32_t active_res, double bandwidth,
                              double* bubble);

/* Bandwidth predictor of Sec. 3.3.1: size of the last chunk over its transmission
 * delay.  Returns -1 unless both are finite and > 0. */
double kvc_est_bandwidth(double last_chunk_size, double last_transmission_delay);

/* A resolution is a tile grid (Sec. 3.2.1 step 2, Sec. 3.3.1: changing the
 * tensor-to-frame layout changes the frame size).  Sets tiles_x = width / tile_w
 * and tiles_y = height / tile_h (integer division, at least 1 each) in *layout,
 * so that a frame is the largest whole-tile picture inside width x height pixels,
 * and validates the result.  The same KV packed under two such layouts restores
 * to the same tensors. */
kvc_status kvc_layout_set_resolution(kvc_layout* layout, int32_t width, int32_t height);

/* Static, never-freed description of a status code. */
/* ---- Intra-frame tiling search (Sec. 3.2.2) -------------------------------
 * The paper fixes the tile by enumerating the tilings its three rules leave
 * and measuring the size of the encoded video of each.  The encoder is outside
 * this library, so the search offered here scores a candidate by a codec-free
 * proxy instead: the first-order entropy of the residuals a predictive coder
 * would store, for the predictors a video codec has.  It ranks tilings; it does
 * not reproduce the paper's compression ratios. */

/* Residuals counted per plane sequence p[f][y][x] (the F frames of one
 * (chunk, kind, layer); arithmetic modulo 256; pixels outside the plane read 0). */
typedef enum {
  KVC_RES_LEFT = 0,      /* p[f][y][x] - p[f][y][x-1]            every frame   */
  KVC_RES_UP = 1,        /* p[f][y][x] - p[f][y-1][x]            every frame   */
  KVC_RES_TIME = 2,      /* t = p[f][y][x] - p[f-1][y][x]        frames f >= 1 */
  KVC_RES_TIME_LEFT = 3, /* t[f][y][x] - t[f][y][x-1]            frames f >= 1 */
  KVC_RES_TIME_UP = 4    /* t[f][y][x] - t[f][y-1][x]            frames f >= 1 */
} kvc_residual;
#define KVC_N_RESIDUALS 5

/* Bytes of the histogram array of n_chunks chunks:
 * uint64 [n_chunks][2][L][KVC_N_RESIDUALS][256]; (size_t)-1 on a bad argument. */
size_t kvc_residual_histograms_size(const kvc_layout* layout, int64_t n_chunks);

/* Counts the residuals of every plane sequence of packed chunks (Sec. 3.2.2:
 * the evaluation step of the tiling search, with the proxy above in place of
 * the encoder).
 *   frames   DEVICE in : n_chunks chunk sections as written by kvc_pack
 *   d_hist   DEVICE out: uint64 [n_chunks][2][L][KVC_N_RESIDUALS][256], every
 *            entry written (no need to clear it); 8-byte aligned
 *   hist_cap capacity of d_hist in bytes; too small -> KVC_ERR_BUFFER_TOO_SMALL
 * KVC_ERR_UNSUPPORTED if one plane sequence has 2^32 pixels or more. */
kvc_status kvc_residual_histograms(const kvc_layout* layout, const uint8_t* frames, int64_t n_chunks,
                                   uint64_t* d_hist, size_t hist_cap, void* stream);

/* Cost in bits of n_chunks chunks from their residual histograms (HOST
 * arithmetic in double).  With H(k) the entropy -sum (n_i/N) log2 (n_i/N) of
 * histogram k of a plane sequence and P = Hp*W pixels per plane, a sequence costs
 *   P * min(H(LEFT), H(UP)) + (F-1) * P * min(H(TIME), H(TIME_LEFT), H(TIME_UP)):
 * the first frame of a group has nothing to predict from in time, the others
 * take their cheapest predictor.  Returns the sum over all sequences, or a
 * negative value on a bad argument.
 *   hist  HOST in: the array kvc_residual_histograms wrote, copied to the host */
double kvc_proxy_cost_bits(const kvc_layout* layout, const uint64_t* hist, int64_t n_chunks);

/* The tilings left by rules i-iii of Sec. 3.2.2 for H heads of D elements:
 * head_num = h1*h2 and head_dim = d1*d2 with all four powers of two, tile
 * (h1*d1, h2*d2), tile_seg = d2 >= 8 (an 8-element atom of the kernels stays in
 * one row).  Writes up to `cap` candidates in the order h1 ascending, then d1
 * ascending, and returns how many there are (which may exceed cap); -1 on a bad
 * argument.  HOST. */
int32_t kvc_tile_candidates(int32_t num_kv_heads, int32_t head_dim, int32_t* tile_h, int32_t* tile_w,
                            int32_t* tile_seg, int32_t cap);

/* Measurement aid, not a step of the paper's path: a streaming copy with the byte
 * ratio of restore (8 bytes read and 16 written per lane).  The benchmark runs it
 * to show what the part delivers for sequential output and for output cut into
 * pieces that land in a given order, and as the copy of known size that profiler
 * byte counters are scaled by.
 *   d_src        DEVICE in : out_bytes / 2 bytes, 8-byte aligned
 *   d_dst        DEVICE out: out_bytes bytes, 16-byte aligned; every byte written
 *                when the map is a permutation
 *   d_piece_map  DEVICE in, may be NULL: piece i of the output (piece_bytes each,
 *                in source order) is written at piece position d_piece_map[i];
 *                entries must be < out_bytes / piece_bytes (not checked: they
 *                are device memory).  NULL: sequential output.
 *   piece_bytes  a power of two, 32768 .. 2^30, dividing out_bytes
 *   wg_bytes     output bytes one workgroup moves in one shot: 4096 or 32768
 *   shape        0, or KVC_PROBE_* bits; any bit needs wg_bytes 4096 and out_bytes
 *                a multiple of 32768
 * Output vector j (16 bytes, source order) is {x, y, x ^ y, s}, (x, y) being source
 * vector s (8 bytes); s = j unless KVC_PROBE_LINE_READS pairs them otherwise. */
enum {
  /* The 8 workgroups that write one 32 KB run of the output run on one XCD
   * (workgroups go to the XCDs round-robin) instead of one on each. */
  KVC_PROBE_ONE_XCD_PER_PIECE = 1,
  /* A workgroup reads its 2 KB as 16 lines of 128 bytes 1 KB apart, the way the
   * codes of two tokens lie in a frame of (8,128) tiles, 8 tiles wide (Sec. 3.2.1
   * step 3): workgroup 8k+m reads lines m, m+8, .. of the 16 KB its group of 8
   * reads together; s = (j / 2048) * 2048 + (j / 256 % 8 + 8 * (j % 256 / 16)) * 16 + j % 16. */
  KVC_PROBE_LINE_READS = 2
};
kvc_status kvc_probe_expand(const void* d_src, void* d_dst, size_t out_bytes, const uint32_t* d_piece_map,
                            size_t piece_bytes, int32_t wg_bytes, int32_t shape, void* stream);

const char* kvc_status_str(kvc_status status);

/* Identifier of what this binary was built from: a hash of the library's
 * sources, this header and the compiler flags, fixed at build time ("unknown"
 * for a build that did not pass one).  Lets a test run detect a stale binary.
 * HOST; returns a static string. */
const char* kvc_build_id(void);

#ifdef __cplusplus
}
#endif
#endif /* KVC_H */
