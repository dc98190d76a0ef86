// Kernel parameter blocks and the host-side launch functions of libkvc.
#pragma once

#include <hip/hip_runtime.h>

#include "kvc_common.h"

namespace kvc {

struct RestoreParams {
  Geo g;
  const uint8_t* frames;  // chunk sections
  const float* meta;      // chunk sections
  int64_t n_tokens;       // tokens held by `frames`
  int32_t n_chunks;
  int32_t tb;             // tokens per workgroup (0: library default)
  int32_t tbc;            // token blocks per chunk
  int32_t tpp;            // tokens per pass of a workgroup = threads / apt
  uint32_t n_units;       // frame call: fm_count * 3 * tbc workgroups with work
  uint32_t units_per_xcd;
  FastDiv dtbc, dL;       // unit -> (token block, chunk), row -> (kind, layer)
  uint32_t row_units;     // chunk call: token blocks of one (kind, layer) over all chunks
  FastDiv drpx;           // ... and the share of one XCD
  // "rows" body: a wave reads runs of 512 bytes of one plane row, i.e. one row of rows_q = 512 / tw neighbouring
  // tiles; a workgroup (th waves) takes rows_trw rows of tiles, in all F frames (chunk call) or in one (frame call)
  int32_t rows_body, rows_q, rows_lat;  // lat: log2 of the atoms of a tile row
  int32_t rows_trw, rows_tile_rows;     // rows of tiles per workgroup; rows of tiles that hold tokens
  FastDiv dnf, dpr;                     // frames a unit covers (F or 1); passes per row of tiles = that * TX / q
  int32_t host_frames;    // `frames` is host memory mapped into the device: prefer the "rows" body
  FastDiv dapt;           // atoms per token
  FastDiv dwpt;           // waves per token (apt / 64) when apt is a multiple of 64
  uint32_t frame_stride;     // bytes from a frame to the next of the same layer group: 3 planes (0 for a frame call)
  // frame call: `frames` holds fm_count consecutive frames (three planes each), the first being
  // frame number fm_first = (kind * LG + layer group) * F + frame index of its chunk
  int32_t frame_mode, fm_first, fm_count;
  // ... of which the first fm_count1 are at `frames`; the others, if any, are a second run of consecutive frames
  // that starts with frame number fm_first2 at `frames2`
  int32_t fm_count1, fm_first2;
  const uint8_t* frames2;
  FastDiv dLG;
  // Where the pairs of (kind, layer l) start: meta + chunk * meta_floats + moff[kind] + (l - meta_l0) * pairs per
  // layer * 2 floats.  A whole chunk section has meta_l0 = 0 and the section's own offsets (set by launch_restore
  // unless meta_sliced); a frame call may bring only the layers of its layer group.
  int32_t meta_sliced, meta_l0;
  int64_t moff[2];
  uint32_t tile_row_stride;  // bytes from a row of tiles to the next: th * W
  // contiguous destination
  uint16_t* out;
  int64_t ls, ks, ts;
  // paged destination
  void* const* layer_cache;
  const int32_t* table;
  int64_t num_blocks;
  FastDiv dbs;            // block size
  int64_t first_token;
  uint32_t* err;
};

// Enqueues the fused unpack + dequantize + placement kernel.
kvc_status launch_restore(RestoreParams p, bool paged, hipStream_t stream);

struct PackParams {
  Geo g;
  const uint16_t* kv;
  int64_t ls, ks, ts;
  int64_t n_tokens;
  int32_t n_chunks;
  uint8_t* frames;
  float* meta;
  // workgroups of per-token kinds: blocks of tb token positions
  int32_t tb, tbc, tpp;
  FastDiv dapt;
  int32_t n_kinds_tok;
  int32_t kinds_tok[2];
  // workgroups of per-channel kinds: strips of channels
  int32_t strip_atoms;    // atoms (8 channels each) per strip, a power of two <= 16
  int32_t n_strips;
  int32_t rows;           // token rows per pass = threads / strip_atoms
  uint32_t pass_step;     // bytes the code offset of a thread grows per pass, 0 if that is not a constant
  int32_t n_kinds_ch;
  int32_t resident;       // per-channel strips are held in registers (one read of the input)
  int32_t kinds_ch[2];
  // token positions of the tile rows a token can fall into: chunks of T tokens, and the call's last chunk
  int32_t positions_full, positions_last;
  // zero-fill workgroups: planes of layers beyond L, then unused tile rows of full chunks, then of the last chunk
  uint32_t pieces_plane, pieces_tail_full, pieces_tail_last;
  uint32_t n_zero_pad, n_zero_full, n_units_zero;
  // work units of the three kinds of workgroup and their share per XCD
  uint32_t n_units_ch, n_units_tok;
  uint32_t ch_per_xcd, tok_per_xcd, zero_per_xcd;
  uint32_t units_per_xcd;
};

// Host-side plan of a pack launch: which body the per-channel kinds take, block and grid
// shape.  Fills the derived fields of `p` (geometry, strides and n_tokens must be set).
kvc_status plan_pack(PackParams& p, int* threads_out);

// Enqueues statistics + quantize + layout for every kind, plus the zero fill of
// unused planes and tile positions.
kvc_status launch_pack(PackParams p, hipStream_t stream);

struct ScoreParams {
  Geo g;
  const uint8_t* frames;  // chunk sections
  int32_t n_chunks;
  uint64_t* hist;         // [n_chunks][2][L][KVC_N_RESIDUALS][256]
  FastDiv dL;             // stream -> (chunk, kind), layer
};

// Enqueues the residual-histogram kernel of the tiling proxy: one workgroup per (chunk, kind, layer).
kvc_status launch_residual_histograms(ScoreParams p, hipStream_t stream);

// Enqueues the reference expand copy (measurement aid): out_bytes / 2 bytes of src -> out_bytes of dst, piece i
// of 2^log2_piece output bytes going to position piece_map[i] (nullptr: in place); wg_bytes is 4096 or 32768;
// shape: KVC_PROBE_* bits (4 KB workgroups, a multiple of 8 of them).
kvc_status launch_probe_expand(const void* src, void* dst, size_t out_bytes, const uint32_t* piece_map, uint32_t log2_piece,
                               int32_t wg_bytes, int32_t shape, hipStream_t stream);

}  // namespace kvc
