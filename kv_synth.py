"""Seeded synthetic KV tensors and the workload shapes they come in.

This module only makes inputs: it holds none of the method's arithmetic (no
quantizer, no layout) and is the one piece shared by the GPU tests, the CPU
oracle tests and the benchmark.

Value recipe (stands in for KV caches of real long-context prompts, which need
trained weights and datasets): for every channel (kind, layer, head, dim) a
standard deviation sigma_c is drawn log-uniformly from [0.1, 4]; with
probability 0.01 the channel is an outlier and sigma_c is multiplied by 10;
values are i.i.d. N(0, sigma_c) over tokens, rounded to fp16 / bf16.
"""
import math
from dataclasses import dataclass

import torch

BASE_SEED = 2602_09725


@dataclass(frozen=True)
class Workload:
    name: str
    index: int          # position in the list of benchmark configurations
    L: int
    H: int
    D: int
    n_tokens: int
    dtype: str          # "f16" | "bf16"
    T: int = 2048       # tokens per chunk
    th: int = 8         # tile (Sec. 3.2.2: (8,128) is the tile found for H=8, D=128)
    tw: int = 128
    TX: int = 8         # tile grid: 8 x 64 positions -> F = 4 frames per group
    TY: int = 64
    block_size: int = 16
    paged: bool = False

    @property
    def C(self):
        return self.H * self.D

    @property
    def n_chunks(self):
        return (self.n_tokens + self.T - 1) // self.T

    @property
    def n_logical_blocks(self):
        return (self.n_tokens + self.block_size - 1) // self.block_size

    @property
    def torch_dtype(self):
        return torch.float16 if self.dtype == "f16" else torch.bfloat16

    @property
    def seed(self):
        return BASE_SEED + self.index


WORKLOADS = {
    "tiny": Workload("tiny", 0, L=2, H=8, D=128, n_tokens=2048, dtype="f16"),
    "llama3_8b_8k": Workload("llama3_8b_8k", 1, L=32, H=8, D=128, n_tokens=8192, dtype="f16"),
    "llama3_8b_32k_paged": Workload("llama3_8b_32k_paged", 2, L=32, H=8, D=128, n_tokens=32768, dtype="f16", paged=True),
    "yi34b_80k_paged": Workload("yi34b_80k_paged", 3, L=60, H=8, D=128, n_tokens=80000, dtype="bf16", paged=True),
    "llama3_8b_32k_pipeline": Workload("llama3_8b_32k_pipeline", 4, L=32, H=8, D=128, n_tokens=32768, dtype="f16", paged=True),
    # not one of the benchmark configurations: the paper's own chunking (Sec. 4 item (1): 10K-token chunks) on a
    # 1080P frame, 1920 x 1080 pixels = 15 x 135 tiles of (8,128), F = 6; three chunks
    "llama3_8b_30k_chunk10k": Workload("llama3_8b_30k_chunk10k", 5, L=32, H=8, D=128, n_tokens=30720, dtype="f16",
                                       T=10240, TX=15, TY=135, paged=True),
}


def channel_sigmas(L, C, gen, device):
    """sigma for every (layer, kind, channel): log-uniform in [0.1, 4], 1 % of channels x10."""
    u = torch.rand((L, 2, C), generator=gen, device=device, dtype=torch.float32)
    sigma = torch.exp(math.log(0.1) + u * (math.log(4.0) - math.log(0.1)))
    outlier = torch.rand((L, 2, C), generator=gen, device=device, dtype=torch.float32) < 0.01
    return torch.where(outlier, sigma * 10.0, sigma)


def make_kv(L, H, D, n_tokens, dtype, seed, device="cpu"):
    """Returns a contiguous [L][2][n_tokens][H][D] tensor of the given torch dtype."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    C = H * D
    sigma = channel_sigmas(L, C, gen, device)
    kv = torch.empty((L, 2, n_tokens, H, D), dtype=dtype, device=device)
    for l in range(L):  # one layer at a time bounds the fp32 temporary
        z = torch.randn((2, n_tokens, C), generator=gen, device=device, dtype=torch.float32)
        kv[l] = (z * sigma[l].unsqueeze(1)).to(dtype).view(2, n_tokens, H, D)
    return kv


def make_workload_kv(w: Workload, device="cpu", n_tokens=None):
    return make_kv(w.L, w.H, w.D, w.n_tokens if n_tokens is None else n_tokens, w.torch_dtype, w.seed, device)


def make_block_table(n_logical, num_blocks, seed, device="cpu"):
    """Seeded random injection logical block -> physical block (a permutation when
    num_blocks == n_logical, else a random subset of the physical blocks)."""
    gen = torch.Generator(device="cpu")
    gen.manual_seed(seed)
    perm = torch.randperm(num_blocks, generator=gen)[:n_logical].to(torch.int32)
    return perm.to(device)


def to_u16(t: torch.Tensor):
    """numpy uint16 view of a CPU fp16 / bf16 tensor (bit patterns)."""
    import numpy as np

    return t.contiguous().view(torch.int16).numpy().view(np.uint16)


def _smooth_along_dim(z, width):
    """Moving average of `width` neighbours along the last axis (circular), rescaled to unit variance."""
    acc = torch.zeros_like(z)
    for s in range(width):
        acc += torch.roll(z, shifts=s, dims=-1)
    return acc / math.sqrt(width)


def make_kv_correlated(L, H, D, n_tokens, dtype, seed, device="cpu", rho=0.8, mean_power=0.5, head_share=0.5):
    """Token-correlated stand-in for a real KV cache, for the tiling search (Sec. 3.2.2).

    The i.i.d. recipe of make_kv has no structure a predictive coder could use, so every tiling would look alike.
    Here, for every (layer, kind), with sigma_c as in make_kv:
        x[t, h, d] = sigma_c * ( m[h, d] + sqrt(head_share) * g[h, d] * a[t, h] + sqrt(1 - head_share) * e[t, h, d] )
      m : per-channel mean, variance mean_power, smooth along d inside a head (8-tap moving average of white noise),
          independent between heads -- channel magnitudes persist over tokens, as in real KV caches;
      a : one AR(1) series per head (coefficient rho, unit variance): what the elements of a head have in common;
      g : loading of the head's series on its elements, +-1 with a sign that is smooth along d;
      e : one AR(1) series per element (coefficient rho, unit variance).
    With rho = 0.8 and mean_power = 0.5 the correlation over channels between the tensors of consecutive tokens is
    about (0.5 + 0.8) / 1.5 = 0.87, the similarity the paper reports along the token axis (Appx A.1).
    Returns [L][2][n_tokens][H][D] of the given torch dtype.  No arithmetic of the method is involved."""
    gen = torch.Generator(device=device)
    gen.manual_seed(seed)
    C = H * D
    sigma = channel_sigmas(L, C, gen, device)                                  # [L][2][C]

    def randn(*shape):
        return torch.randn(shape, generator=gen, device=device, dtype=torch.float32)

    m = _smooth_along_dim(randn(L, 2, H, D), 8) * math.sqrt(mean_power)
    g = torch.sign(_smooth_along_dim(randn(L, 2, H, D), 16))
    g = torch.where(g == 0, torch.ones_like(g), g)
    kv = torch.empty((L, 2, n_tokens, H, D), dtype=dtype, device=device)
    sa, se = math.sqrt(head_share), math.sqrt(1.0 - head_share)
    sig = sigma.view(L, 2, H, D)
    # AR(1) in blocks of B tokens: x[t0 + k] = rho^(k+1) x[t0 - 1] + sum_{j <= k} rho^(k-j) * innov * z[t0 + j], i.e. one
    # lower-triangular Toeplitz product per block instead of one step per token
    B = 64
    k = torch.arange(B, device=device, dtype=torch.float32)
    tri = torch.tril(rho ** (k[:, None] - k[None, :]).clamp(min=0)) * math.sqrt(1.0 - rho * rho)   # [B][B]
    carry = (rho ** (k + 1)).view(B, 1, 1, 1, 1)
    a_prev = randn(L, 2, H, 1)       # state before the first token: a draw from the stationary distribution
    e_prev = randn(L, 2, H, D)
    for t0 in range(0, n_tokens, B):
        nb = min(B, n_tokens - t0)
        a = carry[:nb] * a_prev + torch.einsum("kj,jlchd->klchd", tri[:nb, :nb], randn(nb, L, 2, H, 1))
        e = carry[:nb] * e_prev + torch.einsum("kj,jlchd->klchd", tri[:nb, :nb], randn(nb, L, 2, H, D))
        a_prev, e_prev = a[-1], e[-1]
        kv[:, :, t0:t0 + nb] = (sig * (m + sa * g * a + se * e)).to(dtype).permute(1, 2, 0, 3, 4)
    return kv
