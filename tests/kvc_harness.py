"""Shared plumbing of the GPU parity tests: runs the HIP path through the C ABI
binding and the CPU oracle on the same seeded inputs.  Holds no arithmetic of
the method: it only allocates, calls and compares."""
import ctypes
import sys

import numpy as np
import torch

import kv_synth
import paper_2602_09725_amd as kvc
from oracle import kvco_py as oracle

POISON = 0x7BAD  # fp16 / bf16 bit pattern no restored test value takes by accident


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def layouts(L, H, D, dtype, T, th, tw, TX, TY, k_mode=0, v_mode=1, seg=0):
    """(GPU layout, oracle layout) with the same geometry; dtype is 'f16' | 'bf16'; seg = d2 of a two-level tile."""
    dt = 0 if dtype == "f16" else 1
    return (kvc.Layout(L, H, D, dt, T, th, tw, TX, TY, k_mode, v_mode, seg),
            oracle.make_layout(L, H, D, dt, T, th, tw, TX, TY, k_mode, v_mode, seg))


def workload_layouts(w, L=None):
    return layouts(w.L if L is None else L, w.H, w.D, w.dtype, w.T, w.th, w.tw, w.TX, w.TY)


def stream_handle():
    return torch.cuda.current_stream().cuda_stream


def gpu_pack(glo, kv, n_tokens, guard=4096):
    """kv: contiguous CUDA tensor [L][2][n_tokens][H][D].  Returns (frames, meta) CUDA tensors;
    both are allocated with poison-filled guards that are checked for stray writes."""
    fb, mb, _ = kvc.chunk_sizes(glo)
    nc = (n_tokens + glo.chunk_tokens - 1) // glo.chunk_tokens
    C = glo.num_kv_heads * glo.head_dim
    fbuf = torch.full((guard + nc * fb + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    mbuf = torch.full((guard + nc * mb + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    frames, meta = fbuf[guard:guard + nc * fb], mbuf[guard:guard + nc * mb]
    strides = (2 * n_tokens * C, n_tokens * C, C)
    kvc.kvc_pack(glo, kv.data_ptr(), strides, n_tokens, frames.data_ptr(), nc * fb, meta.data_ptr(), nc * mb,
                 stream_handle())
    torch.cuda.synchronize()
    for buf, n in ((fbuf, nc * fb), (mbuf, nc * mb)):
        assert bool((buf[:guard] == 0xA5).all()) and bool((buf[guard + n:] == 0xA5).all()), "pack wrote outside its buffer"
    return frames, meta.view(torch.float32)


def gpu_restore(glo, frames, meta, n_tokens, torch_dtype, guard=4096):
    C = glo.num_kv_heads * glo.head_dim
    n = glo.num_layers * 2 * n_tokens * C
    buf = torch.full((guard + n + guard,), POISON, dtype=torch.int16, device="cuda")
    out = buf[guard:guard + n]
    strides = (2 * n_tokens * C, n_tokens * C, C)
    kvc.kvc_restore(glo, frames.data_ptr(), meta.data_ptr(), n_tokens, out.data_ptr(), strides, stream_handle())
    torch.cuda.synchronize()
    assert bool((buf[:guard] == POISON).all()) and bool((buf[guard + n:] == POISON).all()), "restore wrote outside"
    return out.view(torch_dtype).view(glo.num_layers, 2, n_tokens, glo.num_kv_heads, glo.head_dim)


class PagedCache:
    """Per-layer paged KV memory [2][num_blocks][block_size][H][D], poison-filled, as an engine would own it."""

    def __init__(self, L, num_blocks, block_size, C, device="cuda"):
        self.L, self.num_blocks, self.block_size, self.C = L, num_blocks, block_size, C
        self.layers = [torch.full((2, num_blocks, block_size, C), POISON, dtype=torch.int16, device=device)
                       for _ in range(L)]
        self.ptrs = torch.tensor([t.data_ptr() for t in self.layers], dtype=torch.int64, device=device)
        self.err = torch.zeros(1, dtype=torch.int32, device=device)

    def numpy_layers(self):
        return [t.cpu().numpy().view(np.uint16) for t in self.layers]


def gpu_restore_paged(glo, frames, meta, first_token, n_tokens, cache: PagedCache, table):
    kvc.kvc_restore_paged(glo, frames.data_ptr(), meta.data_ptr(), first_token, n_tokens, cache.ptrs.data_ptr(),
                          cache.num_blocks, cache.block_size, table.data_ptr(), table.numel(), cache.err.data_ptr(),
                          stream_handle())
    torch.cuda.synchronize()


def oracle_paged(olo, frames_np, meta_np, first_token, n_tokens, L, num_blocks, block_size, C, table_np, caches=None):
    if caches is None:
        caches = [np.full(2 * num_blocks * block_size * C, POISON, dtype=np.uint16) for _ in range(L)]
    err = oracle.restore_paged(olo, frames_np, meta_np, first_token, n_tokens, caches, num_blocks, block_size, table_np)
    return caches, err


def u16(t):
    """numpy uint16 bit view of any 16-bit torch tensor (moved to the host)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def assert_same_bytes(name, got, want):
    got, want = np.asarray(got).reshape(-1), np.asarray(want).reshape(-1)
    assert got.shape == want.shape, (name, got.shape, want.shape)
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError(f"{name}: {bad.size} of {got.size} differ; first at {bad[:8]}: got {got[bad[:8]]} want {want[bad[:8]]}")


def ulp_distance_16(a_bits, b_bits):
    """Distance in units in the last place between two fp16 or two bf16 arrays (as bits)."""
    def key(x):
        x = x.astype(np.int32)
        return np.where(x & 0x8000, 0x8000 - x, x)  # sign-magnitude -> monotone integer
    return np.abs(key(a_bits) - key(b_bits))


def assert_within_one_ulp(name, got_bits, want_bits):
    """The floating-point bar: dequantized values within 1 ulp of the oracle's (they are expected to be identical)."""
    d = ulp_distance_16(np.asarray(got_bits).reshape(-1), np.asarray(want_bits).reshape(-1))
    assert d.max(initial=0) <= 1, f"{name}: max ulp distance {d.max()} at {int(d.argmax())}"
    return int((d != 0).sum())
