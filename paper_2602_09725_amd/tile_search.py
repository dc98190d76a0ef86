"""Intra-frame tiling search (Sec. 3.2.2) on the GPU, with the codec-free proxy in place of the encoder.

For every tiling the three rules leave (kvc_tile_candidates) the same KV tensor is packed at one frame
resolution (kvc_pack), its residual histograms are counted (kvc_residual_histograms) and turned into a cost in
bits (kvc_proxy_cost_bits); candidates are ranked by that cost.  This module only loops and marshals: every
byte of every candidate is produced and counted by the library's kernels.
"""
import torch

from . import kvc


def rank_tiles(kv, n_tokens, dtype, chunk_tokens, frame_width, frame_height, k_mode=kvc.KVC_Q_PER_CHANNEL,
               v_mode=kvc.KVC_Q_PER_TOKEN, candidates=None, stream=None):
    """kv: contiguous CUDA tensor [L][2][n_tokens][H][D] (fp16 or bf16 bits); dtype: kvc.KVC_F16 | kvc.KVC_BF16.
    Every candidate is packed into frames of frame_width x frame_height pixels (whole tiles inside it).
    Returns a list of dicts sorted by cost: tile_h, tile_w, tile_seg, tile_grid, frames_per_group, cost_bits,
    bits_per_element (cost over the number of KV elements)."""
    L, two, n, H, D = kv.shape
    assert two == 2 and n == n_tokens and kv.is_cuda and kv.is_contiguous()
    C = H * D
    sh = (stream or torch.cuda.current_stream()).cuda_stream
    strides = (2 * n_tokens * C, n_tokens * C, C)
    n_chunks = (n_tokens + chunk_tokens - 1) // chunk_tokens
    rows = []
    for th, tw, seg in (candidates or kvc.tile_candidates(H, D)):
        lo = kvc.Layout(L, H, D, dtype, chunk_tokens, th, tw, 1, 1, k_mode, v_mode, seg)
        if kvc.layout_set_resolution(lo, frame_width, frame_height) != 0:
            continue
        fb, mb, F = kvc.chunk_sizes(lo)
        frames = torch.empty(n_chunks * fb, dtype=torch.uint8, device=kv.device)
        meta = torch.empty(n_chunks * mb, dtype=torch.uint8, device=kv.device)
        hbytes = kvc.residual_histograms_size(lo, n_chunks)
        hist = torch.empty(hbytes // 8, dtype=torch.int64, device=kv.device)
        kvc.kvc_pack(lo, kv.data_ptr(), strides, n_tokens, frames.data_ptr(), frames.numel(), meta.data_ptr(),
                     meta.numel(), sh)
        kvc.kvc_residual_histograms(lo, frames.data_ptr(), n_chunks, hist.data_ptr(), hbytes, sh)
        host = hist.cpu()   # synchronizes with the stream the work was enqueued on
        cost = kvc.proxy_cost_bits(lo, host.data_ptr(), n_chunks)
        rows.append({"tile_h": th, "tile_w": tw, "tile_seg": seg, "tile_grid": [lo.tiles_x, lo.tiles_y],
                     "frames_per_group": F, "frame_bytes_per_chunk": fb, "cost_bits": cost,
                     "bits_per_element": cost / (L * 2 * n_tokens * C)})
    rows.sort(key=lambda r: r["cost_bits"])
    return rows
