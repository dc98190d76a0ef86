"""GPU parity of the tiling-search proxy (Sec. 3.2.2): residual histograms of packed chunks against
oracle/residuals.py, bit for bit (integer counts), and the ranking harness against the oracle's costs."""
import numpy as np
import pytest
import torch

import kv_synth
import kvc_harness as hz
from kvc_harness import oracle
from oracle import residuals as R

pytestmark = pytest.mark.gpu

TD = {"f16": torch.float16, "bf16": torch.bfloat16}


@pytest.fixture(scope="module", autouse=True)
def _lib(kvc_lib):
    assert torch.cuda.is_available(), "these tests need the GPU"
    return kvc_lib


def gpu_histograms(glo, frames, n_chunks, guard=64):
    kvc = hz.kvc
    need = kvc.residual_histograms_size(glo, n_chunks)
    buf = torch.full((guard + need // 8 + guard,), -1, dtype=torch.int64, device="cuda")   # poison: every entry must be written
    kvc.kvc_residual_histograms(glo, frames.data_ptr(), n_chunks, buf[guard:].data_ptr(), need, hz.stream_handle())
    torch.cuda.synchronize()
    assert bool((buf[:guard] == -1).all()) and bool((buf[guard + need // 8:] == -1).all()), "wrote outside its buffer"
    return buf[guard:guard + need // 8].cpu().numpy().view(np.uint64)


CASES = [
    # L, H, D, T, th, tw, seg, TX, TY, n_tokens, dtype
    (4, 2, 16, 24, 4, 8, 0, 2, 3, 24 + 13, "f16"),          # tiny planes (12 x 16), F = 4, pad planes, ragged chunk
    (3, 8, 128, 96, 8, 128, 0, 4, 8, 96 + 50, "bf16"),      # the benchmark tile, F = 3
    (2, 8, 128, 64, 16, 64, 16, 2, 4, 64, "f16"),           # a two-level tile, F = 8
    (1, 1, 8, 5, 1, 8, 0, 1, 1, 5, "f16"),                  # one 8-pixel piece per plane, F = 5
    (5, 4, 64, 30, 2, 128, 0, 5, 6, 30, "f16"),             # F = 1: no temporal residuals at all
    (2, 32, 128, 40, 8, 512, 128, 3, 7, 40 * 2 + 3, "f16"), # wide planes (1536 pixels), three chunks
]


@pytest.mark.parametrize("case", CASES, ids=[f"c{i}" for i in range(len(CASES))])
def test_residual_histograms_equal_the_oracle(case):
    L, H, D, T, th, tw, seg, TX, TY, n, dtype = case
    glo, olo = hz.layouts(L, H, D, dtype, T, th, tw, TX, TY, seg=seg)
    kv = kv_synth.make_kv_correlated(L, H, D, n, TD[dtype], seed=40 + L, device="cuda")
    frames, _ = hz.gpu_pack(glo, kv, n)
    n_chunks = (n + T - 1) // T
    hz.say(f"[case] residual histograms L={L} H={H} D={D} T={T} tile=({th},{tw},seg {seg}) grid=({TX},{TY}) n={n} {dtype}")
    got = gpu_histograms(glo, frames, n_chunks).reshape(n_chunks, 2, L, R.N_RESIDUALS, 256)
    # the oracle counts on the oracle's own frames (which the pack tests tie to the GPU's, and so does this line)
    want_frames, _ = oracle.pack(olo, kv_synth.to_u16(kv.cpu()).reshape(-1), n)
    hz.assert_same_bytes("frames", frames.cpu().numpy(), want_frames)
    want = R.residual_histograms(olo, want_frames, n_chunks)
    hz.assert_same_bytes("histograms", got, want)
    F = oracle.frames_per_group(olo)
    plane = TY * th * TX * tw
    assert int(got[0, 0, 0, R.RES_L].sum()) == F * plane and int(got[0, 1, L - 1, R.RES_TU].sum()) == (F - 1) * plane
    # cost through the C ABI against the oracle's
    cost = hz.kvc.proxy_cost_bits(glo, got.ctypes.data, n_chunks)
    want_cost = R.total_cost_bits(olo, want)
    assert abs(cost - want_cost) <= 1e-12 * max(want_cost, 1.0)


def test_histograms_of_adversarial_planes():
    """Frames that are not a pack result: all 255 (every border residual wraps), a ramp, a checkerboard; bit-exact."""
    L, H, D, T, th, tw, TX, TY = 3, 4, 32, 12, 4, 32, 3, 2
    glo, olo = hz.layouts(L, H, D, "f16", T, th, tw, TX, TY)
    fb = oracle.frame_bytes(olo)
    n_chunks = 3
    frames = np.empty(n_chunks * fb, dtype=np.uint8)
    frames[:fb] = 255
    frames[fb:2 * fb] = np.arange(fb) % 251
    yy = (np.arange(fb) // 7 + np.arange(fb)) % 2
    frames[2 * fb:] = (yy * 200).astype(np.uint8)
    got = gpu_histograms(glo, torch.from_numpy(frames).cuda(), n_chunks).reshape(n_chunks, 2, L, R.N_RESIDUALS, 256)
    hz.assert_same_bytes("histograms", got, R.residual_histograms(olo, frames, n_chunks))


def test_rank_tiles_orders_candidates_like_the_oracle():
    """The search loop on a small model shape: every candidate's cost equals the oracle's for the same tiling, so
    the ranking is the oracle's."""
    from paper_2602_09725_amd import tile_search

    L, H, D, T, n = 3, 4, 32, 64, 64 + 20
    W, Hp = 256, 64      # frame of 256 x 64 pixels: 128 tile positions of 128 elements -> F = 1 ... see below
    kv = kv_synth.make_kv_correlated(L, H, D, n, torch.float16, seed=77, device="cuda")
    rows = tile_search.rank_tiles(kv, n, hz.kvc.KVC_F16, T, W // 2, Hp // 2)   # 32 positions -> F = 2
    cands = hz.kvc.tile_candidates(H, D)
    usable = [c for c in cands if c[1] <= W // 2 and c[0] <= Hp // 2]
    assert len(rows) == len(cands) and len(usable) >= 6
    kv_host = kv_synth.to_u16(kv.cpu()).reshape(-1)
    want = {}
    for th, tw, seg in cands:
        TX, TY = max(1, (W // 2) // tw), max(1, (Hp // 2) // th)
        olo = oracle.make_layout(L, H, D, 0, T, th, tw, TX, TY, seg=seg)
        f, _ = oracle.pack(olo, kv_host, n)
        want[(th, tw, seg)] = R.total_cost_bits(olo, R.residual_histograms(olo, f, 2))
    for r in rows:
        w = want[(r["tile_h"], r["tile_w"], r["tile_seg"])]
        assert abs(r["cost_bits"] - w) <= 1e-12 * w, r
    assert [r["cost_bits"] for r in rows] == sorted(r["cost_bits"] for r in rows)
    hz.say("[case] tile ranking: " + ", ".join(f"({r['tile_h']},{r['tile_w']},{r['tile_seg']}) {r['bits_per_element']:.3f}" for r in rows[:5]))
