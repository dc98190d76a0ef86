"""GPU parity: the HIP path through the C ABI against the CPU oracle, element by
element, on the same seeded inputs.

Bar: frame bytes (codes and zero fill), {scale, min} pairs and paged placement
bit-exact; dequantized fp16 / bf16 values within 1 ulp (asserted), and the
number of values that are not identical is reported (expected 0).
"""
import itertools

import numpy as np
import pytest
import torch

import kv_synth
import kvc_harness as hz
from kvc_harness import oracle

pytestmark = pytest.mark.gpu

TD = {"f16": torch.float16, "bf16": torch.bfloat16}


@pytest.fixture(scope="module", autouse=True)
def _lib(kvc_lib):
    assert torch.cuda.is_available(), "these tests need the GPU"
    return kvc_lib


def full_check(glo, olo, kv, n_tokens, dtype, block_size=None, table_seed=0, spare_blocks=3, tag="", host_frames=False):
    """pack -> compare frames/meta; restore contiguous -> compare; restore paged -> compare placement."""
    hz.say(f"[case] {tag} L={olo.L} H={olo.H} D={olo.D} {dtype} T={olo.T} tile=({olo.th},{olo.tw}) grid=({olo.TX},{olo.TY}) "
           f"modes=({olo.k_mode},{olo.v_mode}) n_tokens={n_tokens} bs={block_size}")
    kv_host = kv_synth.to_u16(kv.cpu()).reshape(-1)
    want_frames, want_meta = oracle.pack(olo, kv_host, n_tokens)
    frames, meta = hz.gpu_pack(glo, kv, n_tokens)
    hz.assert_same_bytes("frames", frames.cpu().numpy(), want_frames)
    hz.assert_same_bytes("meta", meta.cpu().numpy().view(np.uint32), want_meta.view(np.uint32))

    want_out = oracle.restore(olo, want_frames, want_meta, n_tokens)
    out = hz.gpu_restore(glo, frames, meta, n_tokens, TD[dtype])
    neq = hz.assert_within_one_ulp("restore", hz.u16(out), want_out)
    assert neq == 0, f"{neq} restored values differ from the oracle by 1 ulp"

    if block_size:
        C = olo.H * olo.D
        n_logical = (n_tokens + block_size - 1) // block_size
        num_blocks = n_logical + spare_blocks
        table = kv_synth.make_block_table(n_logical, num_blocks, table_seed)
        cache = hz.PagedCache(olo.L, num_blocks, block_size, C)
        hz.gpu_restore_paged(glo, frames, meta, 0, n_tokens, cache, table.cuda())
        want_caches, _ = hz.oracle_paged(olo, want_frames, want_meta, 0, n_tokens, olo.L, num_blocks, block_size, C,
                                         table.numpy())
        assert int(cache.err.item()) == 0
        for l, (got, want) in enumerate(zip(cache.numpy_layers(), want_caches)):
            hz.assert_same_bytes(f"paged layer {l}", got, want)
    if host_frames:
        # the same restores with frames and pairs left in pinned host memory (mapped into the device): tiles
        # narrower than 512 bytes are then read by the body that walks plane rows
        hf = torch.empty(frames.numel(), dtype=torch.uint8, pin_memory=True)
        hm = torch.empty(meta.numel(), dtype=torch.float32, pin_memory=True)
        assert hf.numel() == frames.numel() and hm.numel() * 4 == meta.numel() * meta.element_size()
        hf.copy_(frames)
        hm.copy_(meta)
        torch.cuda.synchronize()
        out = hz.gpu_restore(glo, hf, hm, n_tokens, TD[dtype])
        neq = hz.assert_within_one_ulp("restore from host frames", hz.u16(out), want_out)
        assert neq == 0
        if block_size:
            cache = hz.PagedCache(olo.L, num_blocks, block_size, C)
            hz.gpu_restore_paged(glo, hf, hm, 0, n_tokens, cache, table.cuda())
            assert int(cache.err.item()) == 0
            for l, (got, want) in enumerate(zip(cache.numpy_layers(), want_caches)):
                hz.assert_same_bytes(f"paged layer {l} from host frames", got, want)
    return frames, meta


SMALL = [
    # L, H, D, T, th, tw, TX, TY, n_tokens, block_size      (several tiles, ragged last chunk, pad planes)
    (4, 2, 16, 24, 4, 8, 2, 3, 24 + 13, 4),      # C/8 = 4: many tokens per pass, F = 4
    (3, 3, 128, 40, 3, 128, 3, 5, 40 * 2 + 1, 16),  # C/8 = 48: 240-thread workgroups, one-token last chunk
    (5, 8, 128, 96, 8, 128, 4, 8, 96 + 50, 16),  # the benchmark tile, F = 3
    (2, 8, 128, 64, 16, 64, 2, 4, 64 * 3, 7),    # tile (16,64): rows are half heads; odd block size
    (7, 32, 128, 20, 8, 512, 2, 2, 33, 16),      # tile (8,512): four heads per row; C/8 = 512 threads
    (1, 1, 8, 5, 1, 8, 1, 1, 23, 2),             # smallest shapes: one atom per token, F = 5
    (6, 4, 64, 130, 2, 128, 5, 3, 130 + 77, 32), # non power-of-two F (ceil(130/15) = 9) and grid
]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("modes", [(0, 1), (1, 0), (0, 0), (1, 1)])
@pytest.mark.parametrize("shape", SMALL, ids=[f"s{i}" for i in range(len(SMALL))])
def test_small_geometries(shape, modes, dtype):
    L, H, D, T, th, tw, TX, TY, n, bs = shape
    glo, olo = hz.layouts(L, H, D, dtype, T, th, tw, TX, TY, *modes)
    kv = kv_synth.make_kv(L, H, D, n, TD[dtype], seed=1000 + L * 7 + H, device="cuda")
    full_check(glo, olo, kv, n, dtype, block_size=bs, tag="small")


ROW_RUNS = [
    # L, H, D, T, th, tw, seg, TX, TY, n_tokens, block_size: tiles narrower than 512 bytes in rows of tiles of >= 512
    (4, 8, 128, 96, 8, 128, 0, 4, 8, 96 + 50, 16),       # the benchmark tile, one run per row, F = 3
    (3, 8, 128, 300, 8, 128, 0, 8, 5, 300 * 2 + 7, 16),  # two runs per row, F = 8: 16 passes, two rounds of 8
    (2, 8, 128, 64, 16, 64, 0, 8, 2, 64 + 9, 7),         # tile (16,64): 8 tiles per run, 1024 threads, odd block size
    (5, 8, 128, 50, 4, 256, 0, 2, 9, 50 * 3, 32),        # tile (4,256): 2 tiles per run, 256 threads
    (4, 8, 128, 96, 8, 128, 64, 4, 8, 96 + 50, 16),      # two-level (4,2)x(2,64): a tile row holds halves of two heads
    (2, 4, 128, 70, 8, 64, 64, 8, 3, 70 + 33, 16),       # C = 512, two-level with d2 = 64
    (3, 32, 128, 40, 16, 256, 128, 2, 5, 40 + 11, 16),   # 32 heads: tile (16,256) = (16,2)x(1,128)
]


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("modes", [(0, 1), (1, 0)])
@pytest.mark.parametrize("shape", ROW_RUNS, ids=[f"r{i}" for i in range(len(ROW_RUNS))])
def test_frames_left_in_pinned_host_memory(shape, modes, dtype):
    """Restore, contiguous and paged, with frames and pairs in pinned host memory: chunk calls on these tiles take
    the body whose waves read 512-byte runs along plane rows; same oracle comparison as everywhere else."""
    L, H, D, T, th, tw, seg, TX, TY, n, bs = shape
    glo, olo = hz.layouts(L, H, D, dtype, T, th, tw, TX, TY, modes[0], modes[1], seg=seg)
    assert hz.kvc.layout_validate(glo) == 0
    kv = kv_synth.make_kv(L, H, D, n, TD[dtype], seed=4000 + T + th, device="cuda")
    full_check(glo, olo, kv, n, dtype, block_size=bs, tag="row runs", host_frames=True)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", ROW_RUNS, ids=[f"r{i}" for i in range(len(ROW_RUNS))])
def test_frame_calls_and_in_place_pipelines_on_host_blobs(shape, dtype):
    """Blobs left in pinned host memory: runs of consecutive frames restored in place (random cuts of each chunk's
    frame sequence), and both fetch pipelines with no staging, in both orders -- each against the oracle's paged
    restore of the oracle's own frames."""
    L, H, D, T, th, tw, seg, TX, TY, n, bs = shape
    glo, olo = hz.layouts(L, H, D, dtype, T, th, tw, TX, TY, seg=seg)
    C = H * D
    kvc = hz.kvc
    kv = kv_synth.make_kv(L, H, D, n, TD[dtype], seed=77 + n, device="cuda")
    frames, meta = hz.gpu_pack(glo, kv, n)
    fb, mb, F = kvc.chunk_sizes(glo)
    fs = kvc.frame_size(glo)
    per_chunk = fb // fs
    n_chunks = (n + T - 1) // T
    n_logical = (n_chunks * T + bs - 1) // bs
    nb = n_logical + 1
    tab = kv_synth.make_block_table(n_logical, nb, 8).cuda()
    want_f, want_m = oracle.pack(olo, kv_synth.to_u16(kv.cpu()).reshape(-1), n)
    hz.assert_same_bytes("frames", frames.cpu().numpy(), want_f)
    want_caches, oerr = hz.oracle_paged(olo, want_f, want_m, 0, n, L, nb, bs, C, tab.cpu().numpy())
    assert oerr == 0
    moff = kvc.blob_meta_offset(glo)
    blob_bytes = moff + mb
    blobs = []
    for c in range(n_chunks):
        b = torch.zeros(blob_bytes, dtype=torch.uint8, pin_memory=True)
        b[:fb].copy_(frames[c * fb:(c + 1) * fb])
        b[moff:moff + mb].copy_(meta.view(torch.uint8)[c * mb:(c + 1) * mb])
        blobs.append(b)
    torch.cuda.synchronize()

    def check(cache, what):
        torch.cuda.synchronize()
        assert int(cache.err.item()) == 0
        for l, (got_l, want_l) in enumerate(zip(cache.numpy_layers(), want_caches)):
            hz.assert_same_bytes(f"{what}: layer {l}", got_l, want_l)

    rng = np.random.default_rng(n)
    got = hz.PagedCache(L, nb, bs, C)
    for c, b in enumerate(blobs):
        nt = min(T, n - c * T)
        cuts = sorted(set(rng.integers(1, per_chunk, size=3).tolist())) if per_chunk > 1 else []
        for a, e in zip([0] + cuts, cuts + [per_chunk]):
            kvc.kvc_restore_paged_frames(glo, b.data_ptr() + a * fs, b.data_ptr() + moff, a, e - a, c * T, nt,
                                         got.ptrs.data_ptr(), nb, bs, tab.data_ptr(), tab.numel(), got.err.data_ptr(),
                                         hz.stream_handle())
    check(got, "frame ranges in place")
    chunks = [(b.data_ptr(), blob_bytes, min(T, n - c * T)) for c, b in enumerate(blobs)]
    s_comp = torch.cuda.Stream()
    cache = hz.PagedCache(L, nb, bs, C)
    torch.cuda.synchronize()
    kvc.kvc_fetch_pipeline(glo, chunks, [], 0, cache.ptrs.data_ptr(), nb, bs, tab.data_ptr(), tab.numel(),
                           cache.err.data_ptr(), 0, s_comp.cuda_stream, timed=True)
    check(cache, "chunk pipeline in place")
    # untimed forms return after enqueueing; the caller synchronizes the compute stream
    cache = hz.PagedCache(L, nb, bs, C)
    torch.cuda.synchronize()
    assert kvc.kvc_fetch_pipeline(glo, chunks, [], 0, cache.ptrs.data_ptr(), nb, bs, tab.data_ptr(), tab.numel(),
                                  cache.err.data_ptr(), 0, s_comp.cuda_stream, timed=False) is None
    s_comp.synchronize()
    check(cache, "chunk pipeline in place, untimed")
    cache = hz.PagedCache(L, nb, bs, C)
    torch.cuda.synchronize()
    assert kvc.kvc_fetch_pipeline_frames(glo, chunks, [], 0, [], 0, cache.ptrs.data_ptr(), nb, bs, tab.data_ptr(),
                                         tab.numel(), cache.err.data_ptr(), 0, s_comp.cuda_stream,
                                         order=kvc.KVC_ORDER_LAYER, timed=False) is None
    s_comp.synchronize()
    check(cache, "frame pipeline in place, layer order, untimed")
    for order in (kvc.KVC_ORDER_CHUNK, kvc.KVC_ORDER_LAYER):
        cache = hz.PagedCache(L, nb, bs, C)
        torch.cuda.synchronize()
        ms, gms = kvc.kvc_fetch_pipeline_frames(glo, chunks, [], 0, [], 0, cache.ptrs.data_ptr(), nb, bs, tab.data_ptr(),
                                                tab.numel(), cache.err.data_ptr(), 0, s_comp.cuda_stream, order=order,
                                                timed=True, group_times=True)
        assert gms == sorted(gms) and gms[-1] <= ms + 1e-3
        check(cache, f"frame pipeline in place, order {order}")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("modes", [(0, 1), (0, 0)])
@pytest.mark.parametrize("T", [2560, 3584, 4100])
def test_long_chunks_take_the_two_pass_strip_body(dtype, modes, T):
    """Chunks longer than the 2048 tokens a register-resident strip holds (the paper's chunks are 10K tokens,
    Sec. 4 item (1)): the per-channel kinds then keep the last 3072 tokens of a strip on chip (registers and LDS) and
    stream what comes before twice.  The streamed part is empty (2560), one exact step of its loop (512 tokens),
    two steps and a ragged one (1028); the short last chunk fills the on-chip part only partly."""
    L, H, D, n, bs = 2, 8, 128, T + 333, 16
    glo, olo = hz.layouts(L, H, D, dtype, T, 8, 128, 8, 40, *modes)
    kv = kv_synth.make_kv(L, H, D, n, TD[dtype], seed=T, device="cuda")
    full_check(glo, olo, kv, n, dtype, block_size=bs, tag="long chunk")


PAPER_RESOLUTIONS = {"240P": (426, 240), "480P": (854, 480), "640P": (1138, 640), "1080P": (1920, 1080)}


def test_multi_resolution_versions_of_one_cache():
    """One KV cache packed at the paper's four resolutions (Sec. 3.2.1 step 2 / Sec. 3.3.1: a resolution is a tile
    grid): each version bit-exact against the oracle, and all versions restore to the same tensors with the same
    pairs, since the grid moves tiles around but never changes a quantization group."""
    L, H, D, T, n, bs = 4, 8, 128, 2048, 2048 + 700, 16
    kv = kv_synth.make_kv(L, H, D, n, torch.float16, seed=240480, device="cuda")
    first = None
    for name, (wd, ht) in PAPER_RESOLUTIONS.items():
        glo, _ = hz.layouts(L, H, D, "f16", T, 8, 128, 1, 1)
        assert hz.kvc.layout_set_resolution(glo, wd, ht) == 0
        glo, olo = hz.layouts(L, H, D, "f16", T, 8, 128, glo.tiles_x, glo.tiles_y)
        frames, meta = full_check(glo, olo, kv, n, "f16", block_size=bs, tag=f"resolution {name}")
        out = hz.gpu_restore(glo, frames, meta, n, torch.float16)
        if first is None:
            first = (name, meta.clone(), out.clone())
        else:
            assert torch.equal(meta.view(torch.int32), first[1].view(torch.int32)), f"pairs of {name} != {first[0]}"
            assert torch.equal(out.view(torch.int16), first[2].view(torch.int16)), f"{name} restores differently from {first[0]}"


def random_geometries(count, seed):
    """Seeded random layouts inside the documented limits: any C = H*D up to 8192 with D a power of two, any tile
    th*tw == C with tw a multiple of 8, any tile grid, chunk length, layer count, ragged token count and block size."""
    rng = np.random.default_rng(seed)
    out = []
    while len(out) < count:
        H = int(rng.choice([1, 2, 3, 4, 5, 8, 16, 32]))
        D = int(rng.choice([8, 16, 32, 64, 128, 256]))
        C = H * D
        if C > 8192:
            continue
        tws = [w for w in range(8, C + 1, 8) if C % w == 0]
        tw = int(rng.choice(tws))
        th = C // tw
        TX, TY = int(rng.integers(1, 7)), int(rng.integers(1, 7))
        T = int(rng.integers(1, 40 * TX * TY + 1))
        L = int(rng.integers(1, 8))
        n = int(rng.integers(1, 3 * T + 1))
        F = -(-T // (TX * TY))
        frame_bytes = 2 * ((L + 2) // 3) * F * 3 * TY * th * TX * tw * (-(-n // T))
        if L * 2 * n * C > 4_000_000 or frame_bytes > 64 * 2**20:
            continue
        bs = int(rng.choice([1, 2, 7, 16, 32]))
        modes = (int(rng.integers(0, 2)), int(rng.integers(0, 2)))
        dtype = "f16" if rng.integers(0, 2) == 0 else "bf16"
        out.append((L, H, D, T, th, tw, TX, TY, n, bs, modes, dtype))
    return out


@pytest.mark.parametrize("geo", random_geometries(24, seed=20260209), ids=lambda g: "L%d_H%d_D%d_T%d_t%dx%d_g%dx%d_n%d_b%d" % g[:10])
def test_random_geometries(geo):
    L, H, D, T, th, tw, TX, TY, n, bs, modes, dtype = geo
    glo, olo = hz.layouts(L, H, D, dtype, T, th, tw, TX, TY, *modes)
    assert hz.kvc.layout_validate(glo) == 0
    kv = kv_synth.make_kv(L, H, D, n, TD[dtype], seed=31 * L + H + D + n, device="cuda")
    full_check(glo, olo, kv, n, dtype, block_size=bs, tag="random")


def adversarial_kv(L, H, D, n, dtype):
    """Values that stress the quantizer: constant groups, +-0, extremes, exact ties, subnormals, huge ranges."""
    g = torch.Generator().manual_seed(77)
    kv = torch.randn((L, 2, n, H, D), generator=g, dtype=torch.float32)
    kv[0, :, :, 0, :] = 1.25                      # constant along everything: range 0 for both groupings
    kv[0, :, :, 1, :] = -0.0                      # all negative zero
    kv[0, 0, :, 2, :] = torch.arange(D, dtype=torch.float32) / 4  # per-token: exact quarter steps
    kv[0, 1, :, 2, 0::2] = 0.0                    # +0 / -0 mix
    kv[0, 1, :, 2, 1::2] = -0.0
    kv[0, :, :, 3, :] *= 6e-8 if dtype == torch.float16 else 1e-30   # subnormal fp16 / tiny bf16
    if H > 4:
        kv[0, :, :, 4, :] *= 3e4 if dtype == torch.float16 else 1e30   # close to the largest finite values
        kv[0, :, 0, 4, 0] = 65504.0 if dtype == torch.float16 else 1.5e38   # the range must stay finite in fp32
        kv[0, :, 1, 4, 0] = -65504.0 if dtype == torch.float16 else -1.5e38
    if H > 5:
        # codes land exactly on .5 positions: min 0, max 255 * 2^k, values (j + 0.5) * 2^k
        j = torch.arange(D, dtype=torch.float32) % 255
        row = (j + 0.5) * 0.25
        row[0], row[1] = 0.0, 255 * 0.25
        kv[0, :, :, 5, :] = row
    if L > 1:
        kv[1] = kv[1] * 1e-3 + 7.0                # small range on a large offset
    if dtype == torch.float16:
        kv.clamp_(-65504.0, 65504.0)              # inputs must be finite
    return kv.to(dtype)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("modes", [(0, 1), (1, 0)])
def test_adversarial_values(dtype, modes):
    L, H, D, T, n = 3, 8, 128, 48, 48 + 17
    glo, olo = hz.layouts(L, H, D, dtype, T, 8, 128, 4, 4, *modes)
    kv = adversarial_kv(L, H, D, n, TD[dtype]).cuda()
    full_check(glo, olo, kv, n, dtype, block_size=16, tag="adversarial")


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("modes", [(0, 1), (1, 0)], ids=["Kc_Vt", "Kt_Vc"])
@pytest.mark.parametrize("H,D,h1,d1", [(8, 128, 4, 2), (8, 128, 2, 4), (8, 128, 1, 16), (8, 128, 8, 2), (32, 128, 8, 4),
                                       (4, 64, 2, 8), (6, 16, 3, 2)])
def test_two_level_tiles(H, D, h1, d1, modes, dtype):
    """Sec. 3.2.2: head_num -> (h1, h2), head_dim -> (d1, d2), tile (h1*d1, h2*d2), the members that are not a
    row-major reshape included; pack, restore and paged restore against the oracle, ragged last chunk."""
    h2, d2 = H // h1, D // d1
    th, tw = h1 * d1, h2 * d2
    L, T, TX, TY = 4, 40, 2, 5
    n = T + 13
    glo, olo = hz.layouts(L, H, D, dtype, T, th, tw, TX, TY, modes[0], modes[1], seg=d2)
    kv = kv_synth.make_kv(L, H, D, n, TD[dtype], seed=300 + h1 * 17 + d1, device="cuda")
    full_check(glo, olo, kv, n, dtype, block_size=16, tag=f"two-level tile ({h1},{h2})x({d1},{d2})")


def test_strided_input_and_output():
    L, H, D, T, n = 3, 4, 32, 32, 32 + 9
    C = H * D
    glo, olo = hz.layouts(L, H, D, "f16", T, 4, 32, 2, 4)
    kv = kv_synth.make_kv(L, H, D, n, torch.float16, seed=5, device="cuda")
    ts, ks = 2 * C + 8, (n + 3) * (2 * C + 8)
    ls = 2 * ks + 64
    big = torch.full((L * ls + 64,), float("inf"), dtype=torch.float16, device="cuda")  # gaps must never be read
    view = torch.as_strided(big, (L, 2, n, C), (ls, ks, ts, 1))
    view.copy_(kv.view(L, 2, n, C))
    fb, mb, _ = hz.kvc.chunk_sizes(glo)
    nc = 2
    frames = torch.empty(nc * fb, dtype=torch.uint8, device="cuda")
    meta = torch.empty(nc * mb // 4, dtype=torch.float32, device="cuda")
    hz.kvc.kvc_pack(glo, big.data_ptr(), (ls, ks, ts), n, frames.data_ptr(), nc * fb, meta.data_ptr(), nc * mb,
                    hz.stream_handle())
    f2, m2 = hz.gpu_pack(glo, kv, n)
    torch.cuda.synchronize()
    assert torch.equal(frames, f2) and torch.equal(meta.view(torch.int32), m2.view(torch.int32))
    want_f, want_m = oracle.pack(olo, kv_synth.to_u16(kv.cpu()).reshape(-1), n)
    hz.assert_same_bytes("frames", frames.cpu().numpy(), want_f)
    # strided output: everything between the tokens stays poison
    outbuf = torch.full((L * ls + 64,), hz.POISON, dtype=torch.int16, device="cuda")
    hz.kvc.kvc_restore(glo, frames.data_ptr(), meta.data_ptr(), n, outbuf.data_ptr(), (ls, ks, ts), hz.stream_handle())
    torch.cuda.synchronize()
    want = oracle.restore(olo, want_f, want_m, n).reshape(L, 2, n, C)
    got = torch.as_strided(outbuf, (L, 2, n, C), (ls, ks, ts, 1))
    hz.assert_same_bytes("strided restore", got.cpu().numpy().view(np.uint16), want)
    mask = torch.ones_like(outbuf, dtype=torch.bool)
    torch.as_strided(mask, (L, 2, n, C), (ls, ks, ts, 1)).fill_(False)
    assert bool((outbuf[mask] == hz.POISON).all())


def test_token_major_input_with_a_token_stride_beyond_32_bit_row_offsets():
    """Token-major engine tensors [token][layer][kind][H][D] padded so that 2048 rows x token stride passes 4 GiB:
    kvc_pack must leave the register-resident strips (their row offsets are 32-bit) and still equal the oracle."""
    L, H, D, T, n = 2, 8, 128, 48, 48 + 5
    C = H * D
    glo, olo = hz.layouts(L, H, D, "f16", T, 8, 128, 4, 4)
    ts = 2**32 // (2048 * 2) + 8                      # elements between tokens: 2 MiB + 16 bytes
    ls, ks = 2 * C, C                                  # layers and kinds side by side inside a token row
    assert hz.kvc.pack_plan(glo, (ls, ks, ts))[0] == 0 and hz.kvc.pack_plan(glo, (ls, ks, ts - 16))[0] == 1
    kv = kv_synth.make_kv(L, H, D, n, torch.float16, seed=21, device="cuda")
    big = torch.full(((n - 1) * ts + L * 2 * C,), float("inf"), dtype=torch.float16, device="cuda")
    torch.as_strided(big, (L, 2, n, C), (ls, ks, ts, 1)).copy_(kv.view(L, 2, n, C))
    fb, mb, _ = hz.kvc.chunk_sizes(glo)
    nc = 2
    frames = torch.empty(nc * fb, dtype=torch.uint8, device="cuda")
    meta = torch.empty(nc * mb // 4, dtype=torch.float32, device="cuda")
    hz.kvc.kvc_pack(glo, big.data_ptr(), (ls, ks, ts), n, frames.data_ptr(), nc * fb, meta.data_ptr(), nc * mb,
                    hz.stream_handle())
    torch.cuda.synchronize()
    want_f, want_m = oracle.pack(olo, kv_synth.to_u16(kv.cpu()).reshape(-1), n)
    hz.assert_same_bytes("frames", frames.cpu().numpy(), want_f)
    hz.assert_same_bytes("meta", meta.cpu().numpy().view(np.uint32), want_m.view(np.uint32))


def test_paged_bad_block_ids_and_chunked_calls():
    """Ids outside the cache are skipped and reported; chunk-at-a-time calls with first_token fill the same cache."""
    L, H, D, T = 2, 8, 128, 64
    n, bs = 3 * T + 20, 16
    C = H * D
    glo, olo = hz.layouts(L, H, D, "bf16", T, 8, 128, 4, 4)
    kv = kv_synth.make_kv(L, H, D, n, torch.bfloat16, seed=9, device="cuda")
    frames, meta = hz.gpu_pack(glo, kv, n)
    fb, mb, _ = hz.kvc.chunk_sizes(glo)
    n_logical = (n + bs - 1) // bs
    num_blocks = n_logical + 5
    table = kv_synth.make_block_table(n_logical, num_blocks, 3).clone()
    table[2] = num_blocks       # first id past the cache
    table[7] = -1
    table[n_logical - 1] = 2 ** 31 - 1
    cache = hz.PagedCache(L, num_blocks, bs, C)
    tab = table.cuda()
    for c in range(4):  # one call per chunk
        nt = min(T, n - c * T)
        hz.gpu_restore_paged(glo, frames[c * fb:(c + 1) * fb], meta[c * mb // 4:(c + 1) * mb // 4], c * T, nt, cache, tab)
    assert int(cache.err.item()) == 1
    f_np, m_np = frames.cpu().numpy(), meta.cpu().numpy()
    want, err = hz.oracle_paged(olo, f_np, m_np, 0, n, L, num_blocks, bs, C, table.numpy())
    assert err == 1
    for l, (got, w) in enumerate(zip(cache.numpy_layers(), want)):
        hz.assert_same_bytes(f"paged layer {l}", got, w)
    # a clean table leaves the error word alone
    cache2 = hz.PagedCache(L, num_blocks, bs, C)
    hz.gpu_restore_paged(glo, frames, meta, 0, n, cache2, kv_synth.make_block_table(n_logical, num_blocks, 3).cuda())
    assert int(cache2.err.item()) == 0


def test_empty_input_is_a_no_op():
    glo, _ = hz.layouts(2, 8, 128, "f16", 64, 8, 128, 4, 4)
    sentinel = torch.full((1024,), 0x5A, dtype=torch.uint8, device="cuda")
    kvc = hz.kvc
    kvc.kvc_pack(glo, sentinel.data_ptr(), (0, 0, 1024), 0, sentinel.data_ptr(), 0, sentinel.data_ptr(), 0, hz.stream_handle())
    kvc.kvc_restore(glo, sentinel.data_ptr(), sentinel.data_ptr(), 0, sentinel.data_ptr(), (0, 0, 1024), hz.stream_handle())
    torch.cuda.synchronize()
    assert bool((sentinel == 0x5A).all())


# ------------------------------------------------------------------ benchmark configurations


def test_config_tiny_full():
    w = kv_synth.WORKLOADS["tiny"]
    glo, olo = hz.workload_layouts(w)
    kv = kv_synth.make_workload_kv(w, "cuda")
    full_check(glo, olo, kv, w.n_tokens, w.dtype, block_size=16, tag=w.name)


def test_config_llama3_8b_8k_full():
    w = kv_synth.WORKLOADS["llama3_8b_8k"]
    glo, olo = hz.workload_layouts(w)
    kv = kv_synth.make_workload_kv(w, "cuda")
    full_check(glo, olo, kv, w.n_tokens, w.dtype, block_size=None, tag=w.name)


def chunkwise_check(w, chunk_ids, tag):
    """Full-size run on the GPU in the benchmark's launch configuration (one pack call, one paged restore call
    over the whole sequence), compared with the oracle chunk by chunk to bound host memory: chunk sections are
    independent, so the oracle packs / restores chunk c as a one-chunk problem placed at first_token = c*T."""
    glo, olo = hz.workload_layouts(w)
    C, T, bs = w.C, w.T, w.block_size
    hz.say(f"[case] {tag}: generating {w.L}x2x{w.n_tokens}x{C} {w.dtype}")
    kv = kv_synth.make_workload_kv(w, "cuda")
    frames, meta = hz.gpu_pack(glo, kv, w.n_tokens)
    fb, mb, _ = hz.kvc.chunk_sizes(glo)
    n_logical = w.n_logical_blocks
    table = kv_synth.make_block_table(n_logical, n_logical, w.seed)  # a permutation of all blocks
    cache = hz.PagedCache(w.L, n_logical, bs, C)
    hz.gpu_restore_paged(glo, frames, meta, 0, w.n_tokens, cache, table.cuda())
    assert int(cache.err.item()) == 0
    hz.say(f"[case] {tag}: GPU done, checking chunks {list(chunk_ids)}")
    table_np = table.numpy()
    for c in chunk_ids:
        nt = min(T, w.n_tokens - c * T)
        kv_c = kv[:, :, c * T:c * T + nt].contiguous().cpu()
        want_f, want_m = oracle.pack(olo, kv_synth.to_u16(kv_c).reshape(-1), nt)
        hz.assert_same_bytes(f"frames chunk {c}", frames[c * fb:(c + 1) * fb].cpu().numpy(), want_f)
        hz.assert_same_bytes(f"meta chunk {c}", meta[c * mb // 4:(c + 1) * mb // 4].cpu().numpy().view(np.uint32),
                             want_m.view(np.uint32))
        # oracle restore of this chunk into a private poison cache, then compare the blocks it owns
        want_caches, err = hz.oracle_paged(olo, want_f, want_m, c * T, nt, w.L, n_logical, bs, C, table_np)
        assert err == 0
        b0, b1 = c * T // bs, (c * T + nt + bs - 1) // bs
        phys = torch.from_numpy(table_np[b0:b1].astype(np.int64))
        for l in range(w.L):
            got = cache.layers[l][:, phys.cuda()].cpu().numpy().view(np.uint16)
            want = want_caches[l].reshape(2, n_logical, bs, C)[:, phys.numpy()]
            hz.assert_same_bytes(f"paged chunk {c} layer {l}", got, want)
        hz.say(f"[case] {tag}: chunk {c} ok")
    # properties that hold at any size: every slot of a mapped position was written, the tail of the last block was not
    for l in (0, w.L - 1):
        logical_view = cache.layers[l][:, table.long().cuda()].reshape(2, n_logical * bs, C)
        assert int((logical_view[:, :w.n_tokens] == hz.POISON).all(dim=-1).sum()) == 0
        assert bool((logical_view[:, w.n_tokens:] == hz.POISON).all())
    return kv, frames, meta, cache, table


def test_config_llama3_8b_32k_paged():
    w = kv_synth.WORKLOADS["llama3_8b_32k_paged"]
    chunkwise_check(w, range(w.n_chunks), w.name)


def test_config_yi34b_80k_paged_bf16():
    w = kv_synth.WORKLOADS["yi34b_80k_paged"]
    # all 40 chunks, the 128-token tail included (80000 = 39*2048 + 128); all 60 layers, K and V
    chunkwise_check(w, range(w.n_chunks), w.name)


def test_config_pipeline_matches_single_call():
    """16 pinned host blobs, copy on one stream, restore on another: same cache as one kvc_restore_paged call, and
    every chunk and layer of the cache the pipeline filled is compared with the oracle's restore of the same blobs."""
    w = kv_synth.WORKLOADS["llama3_8b_32k_pipeline"]
    glo, olo = hz.workload_layouts(w)
    C, T, bs = w.C, w.T, w.block_size
    kvc = hz.kvc
    kv = kv_synth.make_workload_kv(w, "cuda")
    frames, meta = hz.gpu_pack(glo, kv, w.n_tokens)
    fb, mb, _ = kvc.chunk_sizes(glo)
    moff = kvc.blob_meta_offset(glo)
    blob_bytes = moff + mb
    assert blob_bytes == 142_868_480
    blobs = []
    for c in range(w.n_chunks):
        b = torch.zeros(blob_bytes, dtype=torch.uint8, pin_memory=True)
        b[:fb].copy_(frames[c * fb:(c + 1) * fb])
        b[moff:moff + mb].copy_(meta.view(torch.uint8)[c * mb:(c + 1) * mb])
        blobs.append(b)
    n_logical = w.n_logical_blocks
    table = kv_synth.make_block_table(n_logical, n_logical, w.seed).cuda()
    ref = hz.PagedCache(w.L, n_logical, bs, C)
    hz.gpu_restore_paged(glo, frames, meta, 0, w.n_tokens, ref, table)
    del kv
    for n_staging in (2, 3):
        cache = hz.PagedCache(w.L, n_logical, bs, C)
        staging = [torch.empty(blob_bytes, dtype=torch.uint8, device="cuda") for _ in range(n_staging)]
        s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        ms = kvc.kvc_fetch_pipeline(glo, [(b.data_ptr(), blob_bytes, T) for b in blobs], [s.data_ptr() for s in staging],
                                    blob_bytes, cache.ptrs.data_ptr(), n_logical, bs, table.data_ptr(), n_logical,
                                    cache.err.data_ptr(), s_copy.cuda_stream, s_comp.cuda_stream, timed=True)
        torch.cuda.synchronize()
        hz.say(f"[case] pipeline n_staging={n_staging}: fetch-to-ready {ms:.2f} ms")
        assert ms > 0 and int(cache.err.item()) == 0
        for l in range(w.L):
            assert torch.equal(cache.layers[l], ref.layers[l]), f"layer {l} differs from the single-call restore"
    # no staging at all: the kernels read the pinned blobs in place (n_staging = 0, one stream)
    cache = hz.PagedCache(w.L, n_logical, bs, C)
    ms = kvc.kvc_fetch_pipeline(glo, [(b.data_ptr(), blob_bytes, T) for b in blobs], [], 0, cache.ptrs.data_ptr(),
                                n_logical, bs, table.data_ptr(), n_logical, cache.err.data_ptr(), 0, s_comp.cuda_stream,
                                timed=True)
    torch.cuda.synchronize()
    hz.say(f"[case] pipeline in place: fetch-to-ready {ms:.2f} ms")
    assert ms > 0 and int(cache.err.item()) == 0
    for l in range(w.L):
        assert torch.equal(cache.layers[l], ref.layers[l]), f"in place: layer {l} differs from the single-call restore"
    # untimed form: returns after enqueueing, caller synchronizes
    cache = hz.PagedCache(w.L, n_logical, bs, C)
    r = kvc.kvc_fetch_pipeline(glo, [(b.data_ptr(), blob_bytes, T) for b in blobs], [s.data_ptr() for s in staging],
                               blob_bytes, cache.ptrs.data_ptr(), n_logical, bs, table.data_ptr(), n_logical,
                               cache.err.data_ptr(), s_copy.cuda_stream, s_comp.cuda_stream, timed=False)
    assert r is None
    s_comp.synchronize()
    torch.cuda.synchronize()
    for l in (0, w.L - 1):
        assert torch.equal(cache.layers[l], ref.layers[l])
    # every chunk of the pipeline's own cache against the oracle, which reads the host blobs the pipeline was given
    oracle_check_cache(w, olo, blobs, fb, moff, mb, table.cpu().numpy(), cache, "chunk pipeline")


def oracle_check_cache(w, olo, blobs, fb, moff, mb, table_np, cache, tag):
    """The oracle restores each chunk from its host blob into a private poison cache; the blocks the chunk owns must
    equal the same blocks of `cache` (a PagedCache filled on the GPU) in all layers, K and V."""
    C, T, bs = w.C, w.T, w.block_size
    n_logical = w.n_logical_blocks
    for c, b in enumerate(blobs):
        nt = min(T, w.n_tokens - c * T)
        blob = b.numpy()
        want_caches, err = hz.oracle_paged(olo, blob[:fb], blob[moff:moff + mb].view(np.float32), c * T, nt, w.L,
                                           n_logical, bs, C, table_np)
        assert err == 0
        phys = torch.from_numpy(table_np[c * T // bs:(c * T + nt + bs - 1) // bs].astype(np.int64))
        for l in range(w.L):
            got = cache.layers[l][:, phys.cuda()].cpu().numpy().view(np.uint16)
            hz.assert_same_bytes(f"{tag}: chunk {c} layer {l}", got,
                                 want_caches[l].reshape(2, n_logical, bs, C)[:, phys.numpy()])
        hz.say(f"[case] {tag}: chunk {c} equals the oracle")


# ------------------------------------------------------------------ frame-wise restoration


def gpu_restore_frame(glo, frame, meta, kind, lg, f, first_token, n_tokens, cache, table):
    hz.kvc.kvc_restore_paged_frame(glo, frame.data_ptr(), meta.data_ptr(), kind, lg, f, first_token, n_tokens,
                                   cache.ptrs.data_ptr(), cache.num_blocks, cache.block_size, table.data_ptr(),
                                   table.numel(), cache.err.data_ptr(), hz.stream_handle())


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [SMALL[0], SMALL[2], SMALL[4], SMALL[6]], ids=["s0", "s2", "s4", "s6"])
def test_frame_restore_each_frame_against_oracle(shape, dtype):
    """Every frame of every chunk through kvc_restore_paged_frame into its own poison cache == the oracle's frame
    restore (bit-exact, poison included); all frames into one cache == the chunk-level call."""
    L, H, D, T, th, tw, TX, TY, n, bs = shape
    glo, olo = hz.layouts(L, H, D, dtype, T, th, tw, TX, TY)
    C = H * D
    kv = kv_synth.make_kv(L, H, D, n, TD[dtype], seed=77 + L, device="cuda")
    frames, meta = hz.gpu_pack(glo, kv, n)
    fb, mb, F = hz.kvc.chunk_sizes(glo)
    fs = hz.kvc.frame_size(glo)
    LG = (L + 2) // 3
    assert fs == oracle.frame_size(olo) and fb == 2 * LG * F * fs
    n_logical = (n + bs - 1) // bs
    nb = n_logical + 2
    table = kv_synth.make_block_table(n_logical, nb, 4)
    tab = table.cuda()
    f_np, m_np = frames.cpu().numpy(), meta.cpu().numpy()
    union = hz.PagedCache(L, nb, bs, C)
    for c in range((n + T - 1) // T):
        nt = min(T, n - c * T)
        meta_c = meta[c * mb // 4:(c + 1) * mb // 4]
        for kind, lg, f in itertools.product((0, 1), range(LG), range(F)):
            off = hz.kvc.frame_offset(glo, kind, lg, f)
            assert off == oracle.frame_start(olo, kind, lg, f)
            frame = frames[c * fb + off: c * fb + off + fs]
            one = hz.PagedCache(L, nb, bs, C)
            gpu_restore_frame(glo, frame, meta_c, kind, lg, f, c * T, nt, one, tab)
            gpu_restore_frame(glo, frame, meta_c, kind, lg, f, c * T, nt, union, tab)
            torch.cuda.synchronize()
            want = [np.full(2 * nb * bs * C, hz.POISON, dtype=np.uint16) for _ in range(L)]
            err = oracle.restore_paged_frame(olo, f_np[c * fb + off: c * fb + off + fs], m_np[c * mb // 4:(c + 1) * mb // 4],
                                             kind, lg, f, c * T, nt, want, nb, bs, table.numpy())
            assert err == 0 and int(one.err.item()) == 0
            for l, (got, w) in enumerate(zip(one.numpy_layers(), want)):
                hz.assert_same_bytes(f"chunk {c} frame ({kind},{lg},{f}) layer {l}", got, w)
    ref = hz.PagedCache(L, nb, bs, C)
    hz.gpu_restore_paged(glo, frames, meta, 0, n, ref, tab)
    for l in range(L):
        assert torch.equal(union.layers[l], ref.layers[l])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("shape", [SMALL[1], SMALL[3], SMALL[5], SMALL[6]], ids=["s1", "s3", "s5", "s6"])
def test_frame_ranges_and_small_frame_pipeline(shape, dtype):
    """Runs of consecutive frames in one launch (random cuts of each chunk's frame sequence) and the frame pipeline
    in both orders with slots of one, a few and all frames, ragged last chunk included: same cache as the
    chunk-level call."""
    L, H, D, T, th, tw, TX, TY, n, bs = shape
    glo, olo = hz.layouts(L, H, D, dtype, T, th, tw, TX, TY)
    C = H * D
    kvc = hz.kvc
    kv = kv_synth.make_kv(L, H, D, n, TD[dtype], seed=99 + n, device="cuda")
    frames, meta = hz.gpu_pack(glo, kv, n)
    fb, mb, F = kvc.chunk_sizes(glo)
    fs = kvc.frame_size(glo)
    per_chunk = fb // fs
    n_chunks = (n + T - 1) // T
    n_logical = (n_chunks * T + bs - 1) // bs
    nb = n_logical + 1
    tab = kv_synth.make_block_table(n_logical, nb, 8).cuda()
    ref = hz.PagedCache(L, nb, bs, C)
    hz.gpu_restore_paged(glo, frames, meta, 0, n, ref, tab)
    # the reference of this test is itself the oracle's result (frames and pairs are bit-exact by the pack tests,
    # and are compared again here)
    want_f, want_m = oracle.pack(olo, kv_synth.to_u16(kv.cpu()).reshape(-1), n)
    hz.assert_same_bytes("frames", frames.cpu().numpy(), want_f)
    want_caches, oerr = hz.oracle_paged(olo, want_f, want_m, 0, n, L, nb, bs, C, tab.cpu().numpy())
    assert oerr == 0
    for l, (got_l, want_l) in enumerate(zip(ref.numpy_layers(), want_caches)):
        hz.assert_same_bytes(f"chunk-level restore layer {l}", got_l, want_l)
    rng = np.random.default_rng(n)
    got = hz.PagedCache(L, nb, bs, C)
    for c in range(n_chunks):
        nt = min(T, n - c * T)
        cuts = sorted(set(rng.integers(1, per_chunk, size=3).tolist())) if per_chunk > 1 else []
        for a, b in zip([0] + cuts, cuts + [per_chunk]):
            kvc.kvc_restore_paged_frames(glo, frames[c * fb + a * fs:].data_ptr(), meta[c * mb // 4:].data_ptr(), a, b - a,
                                         c * T, nt, got.ptrs.data_ptr(), nb, bs, tab.data_ptr(), tab.numel(),
                                         got.err.data_ptr(), hz.stream_handle())
    torch.cuda.synchronize()
    assert int(got.err.item()) == 0
    for l in range(L):
        assert torch.equal(got.layers[l], ref.layers[l]), f"frame ranges: layer {l}"
    moff = kvc.blob_meta_offset(glo)
    blob_bytes = moff + mb
    blobs = []
    for c in range(n_chunks):
        b = torch.zeros(blob_bytes, dtype=torch.uint8, pin_memory=True)
        b[:fb].copy_(frames[c * fb:(c + 1) * fb])
        b[moff:moff + mb].copy_(meta.view(torch.uint8)[c * mb:(c + 1) * mb])
        blobs.append(b)
    chunks = [(b.data_ptr(), blob_bytes, min(T, n - c * T)) for c, b in enumerate(blobs)]
    s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
    LG = (L + 2) // 3
    for order in (kvc.KVC_ORDER_CHUNK, kvc.KVC_ORDER_LAYER):
        msz = kvc.meta_staging_size(glo, order)
        for per_slot, n_fs, n_ms in ((1, 2, 2), (3, 3, 2), (2 * F + 1, 2, 3), (per_chunk + 2, 2, 2)):
            cache = hz.PagedCache(L, nb, bs, C)
            fstage = [torch.empty(per_slot * fs + 256, dtype=torch.uint8, device="cuda") for _ in range(n_fs)]
            mstage = [torch.full((msz + 256,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(n_ms)]
            torch.cuda.synchronize()
            ms, gms = kvc.kvc_fetch_pipeline_frames(glo, chunks, [s.data_ptr() for s in fstage], per_slot * fs + 255,
                                                    [s.data_ptr() for s in mstage], msz, cache.ptrs.data_ptr(), nb, bs,
                                                    tab.data_ptr(), tab.numel(), cache.err.data_ptr(),
                                                    s_copy.cuda_stream, s_comp.cuda_stream, order=order, timed=True,
                                                    group_times=True)
            torch.cuda.synchronize()
            assert ms > 0 and int(cache.err.item()) == 0
            assert len(gms) == LG and all(0 < t <= ms + 1e-3 for t in gms) and gms == sorted(gms)
            for l in range(L):
                assert torch.equal(cache.layers[l], ref.layers[l]), f"order {order} per_slot={per_slot}: layer {l}"
            for m in mstage:  # nothing written behind the stated meta staging size
                assert bool((m[msz:] == 0xEE).all())


def test_restore_reads_frames_from_mapped_pinned_host_memory():
    """The frame pointer may be pinned host memory that is mapped into the device (no staging copy at all)."""
    L, H, D, T, n, bs = 3, 8, 128, 96, 96 + 40, 16
    glo, olo = hz.layouts(L, H, D, "f16", T, 8, 128, 4, 8)
    kv = kv_synth.make_kv(L, H, D, n, torch.float16, seed=12, device="cuda")
    frames, meta = hz.gpu_pack(glo, kv, n)
    host = torch.empty(frames.numel(), dtype=torch.uint8, pin_memory=True)
    host.copy_(frames)
    torch.cuda.synchronize()
    n_logical = (n + bs - 1) // bs
    tab = kv_synth.make_block_table(n_logical, n_logical + 2, 5).cuda()
    ref = hz.PagedCache(L, n_logical + 2, bs, H * D)
    hz.gpu_restore_paged(glo, frames, meta, 0, n, ref, tab)
    got = hz.PagedCache(L, n_logical + 2, bs, H * D)
    hz.gpu_restore_paged(glo, host, meta, 0, n, got, tab)
    for l in range(L):
        assert torch.equal(got.layers[l], ref.layers[l])
    # the pairs from pinned host memory as well
    host_meta = torch.empty(meta.numel(), dtype=torch.float32, pin_memory=True)
    host_meta.copy_(meta)
    torch.cuda.synchronize()
    got2 = hz.PagedCache(L, n_logical + 2, bs, H * D)
    hz.gpu_restore_paged(glo, host, host_meta, 0, n, got2, tab)
    for l in range(L):
        assert torch.equal(got2.layers[l], ref.layers[l])


def test_frame_restore_bad_block_ids():
    L, H, D, T, n, bs = 3, 8, 128, 64, 64, 16
    glo, olo = hz.layouts(L, H, D, "f16", T, 8, 128, 4, 4)
    kv = kv_synth.make_kv(L, H, D, n, torch.float16, seed=3, device="cuda")
    frames, meta = hz.gpu_pack(glo, kv, n)
    fs = hz.kvc.frame_size(glo)
    table = torch.tensor([2, 99, 0, -5], dtype=torch.int32)
    cache = hz.PagedCache(L, 4, bs, H * D)
    gpu_restore_frame(glo, frames[:fs], meta, 0, 0, 0, 0, n, cache, table.cuda())
    torch.cuda.synchronize()
    want = [np.full(2 * 4 * bs * H * D, hz.POISON, dtype=np.uint16) for _ in range(L)]
    err = oracle.restore_paged_frame(olo, frames[:fs].cpu().numpy(), meta.cpu().numpy(), 0, 0, 0, 0, n, want, 4, bs, table.numpy())
    assert err == 1 and int(cache.err.item()) == 1
    for l, (got, w) in enumerate(zip(cache.numpy_layers(), want)):
        hz.assert_same_bytes(f"layer {l}", got, w)


def test_config_frame_pipeline_matches_chunk_restore():
    """Benchmark pipeline workload at frame granularity: a few frame-sized staging slots instead of chunk blobs."""
    w = kv_synth.WORKLOADS["llama3_8b_32k_pipeline"]
    glo, olo = hz.workload_layouts(w)
    C, T, bs = w.C, w.T, w.block_size
    kvc = hz.kvc
    kv = kv_synth.make_workload_kv(w, "cuda")
    frames, meta = hz.gpu_pack(glo, kv, w.n_tokens)
    del kv
    fb, mb, _ = kvc.chunk_sizes(glo)
    moff = kvc.blob_meta_offset(glo)
    blob_bytes = moff + mb
    blobs = []
    for c in range(w.n_chunks):
        b = torch.zeros(blob_bytes, dtype=torch.uint8, pin_memory=True)
        b[:fb].copy_(frames[c * fb:(c + 1) * fb])
        b[moff:moff + mb].copy_(meta.view(torch.uint8)[c * mb:(c + 1) * mb])
        blobs.append(b)
    n_logical = w.n_logical_blocks
    table = kv_synth.make_block_table(n_logical, n_logical, w.seed).cuda()
    ref = hz.PagedCache(w.L, n_logical, bs, C)
    hz.gpu_restore_paged(glo, frames, meta, 0, w.n_tokens, ref, table)
    fs = kvc.frame_size(glo)
    assert fs == 1_572_864
    LG = (w.L + 2) // 3
    for order, per_slot, n_fs, n_ms in ((0, 1, 2, 2), (0, 16, 3, 3), (1, 4, 3, 2), (1, 16, 3, 4)):
        cache = hz.PagedCache(w.L, n_logical, bs, C)
        msz = kvc.meta_staging_size(glo, order)
        fstage = [torch.empty(per_slot * fs, dtype=torch.uint8, device="cuda") for _ in range(n_fs)]
        mstage = [torch.empty(msz, dtype=torch.uint8, device="cuda") for _ in range(n_ms)]
        s_copy, s_comp = torch.cuda.Stream(), torch.cuda.Stream()
        torch.cuda.synchronize()
        ms, gms = kvc.kvc_fetch_pipeline_frames(glo, [(b.data_ptr(), blob_bytes, T) for b in blobs],
                                                [s.data_ptr() for s in fstage], per_slot * fs,
                                                [s.data_ptr() for s in mstage], msz,
                                                cache.ptrs.data_ptr(), n_logical, bs, table.data_ptr(), n_logical,
                                                cache.err.data_ptr(), s_copy.cuda_stream, s_comp.cuda_stream,
                                                order=order, timed=True, group_times=True)
        torch.cuda.synchronize()
        hz.say(f"[case] frame pipeline order={order}, {n_fs} slots of {per_slot} frames, {n_ms} meta slots: "
               f"fetch-to-ready {ms:.2f} ms, first/last group ready {gms[0]:.2f}/{gms[-1]:.2f} ms, "
               f"staging {(n_fs * per_slot * fs + n_ms * msz) / 2**20:.1f} MiB")
        assert ms > 0 and int(cache.err.item()) == 0
        assert gms == sorted(gms) and gms[-1] <= ms + 1e-3
        if order == kvc.KVC_ORDER_LAYER:
            assert gms[0] < ms / 4   # the first of 11 groups is ready long before the last
        else:
            assert gms[0] > ms / 2   # chunk order completes every group only in the last of 16 chunks
        for l in range(w.L):
            assert torch.equal(cache.layers[l], ref.layers[l]), f"layer {l} differs from the chunk-level restore"
    # no staging at all (n_frame_staging = 0): every run of frames is restored by a kernel that reads the blob in place
    for order in (kvc.KVC_ORDER_CHUNK, kvc.KVC_ORDER_LAYER):
        cache = hz.PagedCache(w.L, n_logical, bs, C)
        torch.cuda.synchronize()
        ms, gms = kvc.kvc_fetch_pipeline_frames(glo, [(b.data_ptr(), blob_bytes, T) for b in blobs], [], 0, [], 0,
                                                cache.ptrs.data_ptr(), n_logical, bs, table.data_ptr(), n_logical,
                                                cache.err.data_ptr(), 0, s_comp.cuda_stream, order=order, timed=True,
                                                group_times=True)
        torch.cuda.synchronize()
        hz.say(f"[case] frame pipeline in place, order={order}: fetch-to-ready {ms:.2f} ms, first/last group ready "
               f"{gms[0]:.2f}/{gms[-1]:.2f} ms")
        assert ms > 0 and int(cache.err.item()) == 0
        assert gms == sorted(gms) and gms[-1] <= ms + 1e-3
        if order == kvc.KVC_ORDER_LAYER:
            assert gms[0] < ms / 4
        for l in range(w.L):
            assert torch.equal(cache.layers[l], ref.layers[l]), f"in place, order {order}: layer {l} differs"
    # caller-made events, call returns after enqueueing: once group g's event has fired its layers are complete
    cache = hz.PagedCache(w.L, n_logical, bs, C)
    events = [torch.cuda.Event() for _ in range(LG)]
    for e in events:
        e.record(s_comp)   # torch creates the underlying event at its first record
    torch.cuda.synchronize()
    r = kvc.kvc_fetch_pipeline_frames(glo, [(b.data_ptr(), blob_bytes, T) for b in blobs],
                                      [s.data_ptr() for s in fstage], per_slot * fs, [s.data_ptr() for s in mstage], msz,
                                      cache.ptrs.data_ptr(), n_logical, bs, table.data_ptr(), n_logical,
                                      cache.err.data_ptr(), s_copy.cuda_stream, s_comp.cuda_stream,
                                      order=kvc.KVC_ORDER_LAYER, group_ready_events=[e.cuda_event for e in events],
                                      timed=False)
    assert r is None
    for g in (0, LG // 2, LG - 1):
        events[g].synchronize()
        for l in range(3 * g, min(3 * g + 3, w.L)):
            assert torch.equal(cache.layers[l], ref.layers[l]), f"group {g} event fired before layer {l} was complete"
    s_comp.synchronize()
    torch.cuda.synchronize()
    # the non-blocking form can be captured into a HIP graph (it holds copies, kernels and event edges only, no
    # memset): every replay, with eager work between the replays, gives the cache of the eager call
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=s_copy):
        kvc.kvc_fetch_pipeline_frames(glo, [(b.data_ptr(), blob_bytes, T) for b in blobs],
                                      [s.data_ptr() for s in fstage], per_slot * fs, [s.data_ptr() for s in mstage], msz,
                                      cache.ptrs.data_ptr(), n_logical, bs, table.data_ptr(), n_logical,
                                      cache.err.data_ptr(), s_copy.cuda_stream, s_comp.cuda_stream,
                                      order=kvc.KVC_ORDER_LAYER, timed=False)
        joined = torch.cuda.Event()
        joined.record(s_comp)
        s_copy.wait_event(joined)   # the capture ends on the stream it began on
    torch.cuda.synchronize()
    for rep in range(3):
        for t in cache.layers:
            t.fill_(hz.POISON)      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert int(cache.err.item()) == 0
        for l in range(w.L):
            assert torch.equal(cache.layers[l], ref.layers[l]), f"graph replay {rep}: layer {l}"
    # the cache the last replay filled, chunk by chunk and layer by layer against the oracle
    oracle_check_cache(w, olo, blobs, fb, moff, mb, table.cpu().numpy(), cache, "frame pipeline (graph replay)")


@pytest.mark.parametrize("wg", [4096, 32768])
def test_reference_expand_copy_moves_every_vector_where_the_map_says(wg):
    """The measurement aid kvc_probe_expand: vector j of the source order lands in piece map[j / per_piece] at the
    same offset, with and without a map, whichever XCD its workgroup runs on; with line reads it carries the source
    vector the header's formula pairs it with; nothing outside the destination is written."""
    out_bytes, piece = 3 << 20, 32768
    n_vec, per_piece = out_bytes // 16, piece // 16
    src = torch.randint(-2**31, 2**31 - 1, (n_vec, 2), dtype=torch.int32, device="cuda")
    guard = 1024
    j = torch.arange(n_vec, device="cuda")
    for use_map in (False, True):
        for shape in ((0, 1, 2, 3) if wg == 4096 else (0,)):
            buf = torch.full((guard + n_vec * 4 + guard,), 0x5A5A5A5A, dtype=torch.int32, device="cuda")
            dst = buf[guard:guard + n_vec * 4]
            assert dst.data_ptr() % 16 == 0
            pm = torch.randperm(out_bytes // piece, generator=torch.Generator().manual_seed(3)).to(torch.int32).cuda()
            hz.kvc.kvc_probe_expand(src.data_ptr(), dst.data_ptr(), out_bytes, pm.data_ptr() if use_map else 0, piece, wg,
                                    hz.stream_handle(), shape=shape)
            torch.cuda.synchronize()
            s = j
            if shape & hz.kvc.PROBE_LINE_READS:
                s = (j // 2048) * 2048 + ((j // 256) % 8 + 8 * ((j % 256) // 16)) * 16 + j % 16
                assert torch.equal(torch.sort(s).values, j)   # every source vector is read exactly once
            want = torch.stack([src[s, 0], src[s, 1], src[s, 0] ^ src[s, 1], s.to(torch.int32)], dim=1)
            where = (pm.long()[j // per_piece] * per_piece + j % per_piece) if use_map else j
            got = dst.view(n_vec, 4)[where]
            assert torch.equal(got, want), (use_map, shape)
            assert bool((buf[:guard] == 0x5A5A5A5A).all()) and bool((buf[guard + n_vec * 4:] == 0x5A5A5A5A).all())
