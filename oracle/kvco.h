/*
 * kvco.h -- CPU oracle of the KV pack / restore path of KVCodec (arXiv 2602.09725).
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, scalar C statement of what
 * the path computes, written from the paper; it shares no code, header, table or
 * helper with the GPU library and is linked by the tests, the smoke check and
 * the benchmark's CPU-baseline leg alone.  Nothing in the product may call it.
 *
 * Passages followed
 *   Sec. 3.2 (first paragraph)   KV cache [token, layer, head_num, head_dim] ->
 *                                video [frame, height, width, 3]
 *   Sec. 3.2.1 steps 1-3         three-layer chunks sliced along tokens; T token
 *                                tensors in groups of F; the F tensors of a group
 *                                at one position in F consecutive frames; three
 *                                layers -> three independently coded planes
 *   Sec. 3.2.2 rules i-iii       tile = geometric tiling of the H*D vector, heads
 *                                and in-head order kept: head_num reshaped to
 *                                (h1, h2), head_dim to (d1, d2), tile = (h1*d1,
 *                                h2*d2) (the closing paragraph's (32,128) ->
 *                                (8,4) x (1,128) -> (8,512); tiles (8,512),
 *                                (8,128), (16,64) found there)
 *   Sec. 4 item (1)              tensors become integers before encoding; chunking
 *   Sec. 3.3.2 restoration       frame -> KV tensor -> preallocated paged slots
 *
 * Pins (tests marked "not gpu"): index map against the paper's three worked
 * tiles and rules i-iii, the two-level tilings against numpy's own
 * reshape / transpose / reshape, the temporal-alignment and three-plane statements,
 * brute-force bijection, a layout special case equal to a numpy reshape, the
 * uniform-quantizer error bound, exact extremes, numpy's own float16 rounding,
 * paged placement against a poison-filled cache, the frame-wise restore against
 * the set of tokens and layers a frame carries (Sec. 3.2.1 step 3) and against
 * the chunk-level restore.  Compression ratio, accuracy
 * and TTFT of the paper need a codec, weights and datasets: parity unpinned,
 * and not computed here.
 */
#ifndef KVCO_H
#define KVCO_H
#include <stddef.h>
#include <stdint.h>

typedef struct {
  int32_t L, H, D;      /* layers, KV heads, head_dim                     */
  int32_t dtype;        /* 0 = fp16, 1 = bf16                             */
  int32_t T;            /* tokens per chunk                               */
  int32_t th, tw;       /* tile, th*tw == H*D                             */
  int32_t TX, TY;       /* tile grid of one frame                         */
  int32_t k_mode;       /* 0 = one group per channel per chunk            */
  int32_t v_mode;       /* 1 = one group per (token, head)                */
  int32_t seg;          /* 0: tile = row-major reshape of the H*D vector;
                           d2 > 0: two-level tiling, d2 consecutive elements
                           of one head per tile row                         */
} kvco_layout;

int kvco_check(const kvco_layout* lo);                       /* 0 if consistent */
int64_t kvco_frames_per_group(const kvco_layout* lo);        /* F  */
int64_t kvco_frame_bytes(const kvco_layout* lo);             /* per chunk */
int64_t kvco_meta_floats(const kvco_layout* lo);             /* per chunk, in floats */
int64_t kvco_meta_kind_offset(const kvco_layout* lo, int kind); /* floats from the chunk's meta start */

/* byte offset, inside one chunk's frame section, of element (kind, l, t, h, d) */
int64_t kvco_frame_offset(const kvco_layout* lo, int kind, int l, int64_t t, int h, int d);
/* float offset, inside one chunk's meta section, of the {scale, mn} pair of that element's group */
int64_t kvco_meta_offset(const kvco_layout* lo, int kind, int l, int64_t t, int h, int d);

/* element conversions, exposed so tests can pin them against numpy */
float kvco_widen(uint16_t bits, int dtype);
uint16_t kvco_narrow(float x, int dtype);
/* one group: statistics of xs[0..n) -> scale, mn, inv */
void kvco_group_params(const float* xs, int64_t n, float* scale, float* mn, float* inv);
uint8_t kvco_quantize(float x, float mn, float inv);
float kvco_dequantize(uint8_t code, float scale, float mn);

/* kv: [L][2][n_tokens][H][D] 16-bit words addressed with element strides.
 * frames / meta: ceil(n_tokens/T) chunk sections, fully written. returns 0 on success. */
int kvco_pack(const kvco_layout* lo, const uint16_t* kv, int64_t layer_stride, int64_t kv_stride,
              int64_t token_stride, int64_t n_tokens, uint8_t* frames, float* meta);
int kvco_restore(const kvco_layout* lo, const uint8_t* frames, const float* meta, int64_t n_tokens,
                 uint16_t* kv_out, int64_t layer_stride, int64_t kv_stride, int64_t token_stride);
/* layer_cache[l]: [2][num_blocks][block_size][H][D]. Blocks whose id is out of
 * range are skipped and *err (may be NULL) gets bit 0 set. */
int kvco_restore_paged(const kvco_layout* lo, const uint8_t* frames, const float* meta, int64_t first_token,
                       int64_t n_tokens, uint16_t* const* layer_cache, int64_t num_blocks, int32_t block_size,
                       const int32_t* block_table, int64_t table_len, uint32_t* err);
/* Frame-wise restoration (Sec. 3.3.2): `frame` holds the three planes of (kind, layer group lg,
 * frame index f) of the chunk that starts at sequence position first_token and has n_tokens
 * valid tokens; meta is that chunk's meta section.  Writes the tokens t with t % F == f of the
 * layers 3*lg .. 3*lg+2 that exist. */
int kvco_restore_paged_frame(const kvco_layout* lo, const uint8_t* frame, const float* meta, int kind, int lg, int f,
                             int64_t first_token, int64_t n_tokens, uint16_t* const* layer_cache, int64_t num_blocks,
                             int32_t block_size, const int32_t* block_table, int64_t table_len, uint32_t* err);
int kvco_threads(void); /* threads the chunk/layer loops run on */
const char* kvco_build_id(void); /* hash of the sources and flags this binary was built from */
#endif
