"""Pins of the tiling-proxy oracle (oracle/residuals.py) and of the token-correlated input recipe.  Expected values
are hand-made or closed forms; none comes from the function under test."""
import math

import numpy as np
import torch

import kv_synth
from oracle import kvco_py as oracle
from oracle import residuals as R


def test_hand_made_planes():
    # two frames of a 2 x 3 plane
    p = np.array([[[10, 12, 12], [10, 250, 3]],
                  [[11, 12, 13], [9, 250, 0]]], dtype=np.uint8)
    h = R.stream_histograms(p)
    def hist_of(values):
        out = np.zeros(256, dtype=np.uint64)
        for v in values:
            out[v % 256] += 1
        return out
    # left: first column against 0
    assert np.array_equal(h[R.RES_L], hist_of([10, 2, 0, 10, 240, 9,   11, 1, 1, 9, 241, 6]))
    # up: first row against 0
    assert np.array_equal(h[R.RES_U], hist_of([10, 12, 12, 0, 238, 247,   11, 12, 13, 254, 238, 243]))
    t = [1, 0, 1, 255, 0, 253]
    assert np.array_equal(h[R.RES_T], hist_of(t))
    assert np.array_equal(h[R.RES_TL], hist_of([1, 255, 1, 255, 1, 253]))       # t[x] - t[x-1] per row
    assert np.array_equal(h[R.RES_TU], hist_of([1, 0, 1, 254, 0, 252]))         # second row minus first
    assert [int(x.sum()) for x in h] == [12, 12, 6, 6, 6]


def test_entropy_closed_forms():
    const = np.zeros(256); const[7] = 1000
    assert R.entropy_bits_per_symbol(const) == 0.0
    assert abs(R.entropy_bits_per_symbol(np.full(256, 5)) - 8.0) < 1e-12
    two = np.zeros(256); two[0] = 3; two[255] = 1
    assert abs(R.entropy_bits_per_symbol(two) - (2 - 0.75 * math.log2(3))) < 1e-12
    assert R.entropy_bits_per_symbol(np.zeros(256)) == 0.0


def test_structured_planes_have_the_zero_residuals_they_must():
    rng = np.random.default_rng(1)
    F, Hp, W = 3, 8, 16
    frame = rng.integers(0, 256, size=(Hp, W), dtype=np.uint8)
    rep = np.stack([frame] * F)                          # the same frame again and again
    h = R.stream_histograms(rep)
    assert h[R.RES_T][0] == (F - 1) * Hp * W and h[R.RES_TL][0] == (F - 1) * Hp * W and h[R.RES_TU][0] == (F - 1) * Hp * W
    col = np.broadcast_to(rng.integers(1, 256, size=(F, Hp, 1), dtype=np.uint8), (F, Hp, W))   # constant along x
    h = R.stream_histograms(col)
    assert h[R.RES_L][0] == F * Hp * (W - 1)             # only the border column differs from its (absent) neighbour
    row = np.broadcast_to(rng.integers(1, 256, size=(F, 1, W), dtype=np.uint8), (F, Hp, W))     # constant along y
    h = R.stream_histograms(row)
    assert h[R.RES_U][0] == F * (Hp - 1) * W


def test_temporal_histogram_does_not_depend_on_where_pixels_sit():
    """Any tile keeps a channel at one pixel in all frames (Sec. 3.2.1 step 3), so the temporal residuals are the same
    multiset for every tiling: a permutation of the pixel positions leaves that histogram alone."""
    rng = np.random.default_rng(2)
    p = rng.integers(0, 256, size=(4, 6, 10), dtype=np.uint8)
    perm = rng.permutation(60)
    q = p.reshape(4, 60)[:, perm].reshape(4, 6, 10)
    assert np.array_equal(R.stream_histograms(p)[R.RES_T], R.stream_histograms(q)[R.RES_T])
    assert not np.array_equal(R.stream_histograms(p)[R.RES_L], R.stream_histograms(q)[R.RES_L])


def test_streams_are_the_planes_of_the_layout_and_costs_add_up():
    lo = oracle.make_layout(L=4, H=2, D=16, dtype=0, T=24, th=4, tw=8, TX=2, TY=3)
    F = oracle.frames_per_group(lo)
    assert F == 4
    n_chunks = 2
    fb = oracle.frame_bytes(lo)
    rng = np.random.default_rng(3)
    frames = rng.integers(0, 256, size=n_chunks * fb, dtype=np.uint8)
    hists = R.residual_histograms(lo, frames, n_chunks)
    assert hists.shape == (n_chunks, 2, 4, 5, 256)
    plane = 12 * 16
    # layer 3 of V in chunk 1 is plane 0 of layer group 1: cut it out with the oracle's own index map for element (0, 0)
    base = 1 * fb + oracle.frame_offset(lo, 1, 3, 0, 0, 0)
    seq = np.stack([frames[base + f * 3 * plane: base + f * 3 * plane + plane].reshape(12, 16) for f in range(F)])
    assert np.array_equal(hists[1, 1, 3], R.stream_histograms(seq))
    assert int(hists[0, 0, 0, R.RES_L].sum()) == F * plane and int(hists[0, 0, 0, R.RES_T].sum()) == (F - 1) * plane
    total = R.total_cost_bits(lo, hists)
    assert abs(total - sum(R.stream_cost_bits(lo, hists[c, k, l]) for c in range(2) for k in range(2) for l in range(4))) < 1e-6
    # random bytes cost about 8 bits each, whatever the predictor
    assert 7.0 * n_chunks * 2 * 4 * F * plane < total <= 8.0 * n_chunks * 2 * 4 * F * plane


def test_tile_candidates_are_the_two_level_factorizations():
    c = R.tile_candidates(8, 128)
    assert len(c) == 4 * 5 and len(set(c)) == len(c)
    assert (8, 128, 128) in c and (16, 64, 64) in c          # two of the tiles the paper reports
    assert (8, 512, 128) in R.tile_candidates(32, 128) and len(R.tile_candidates(32, 128)) == 6 * 5
    for th, tw, seg in c:
        assert th * tw == 1024 and 128 % seg == 0 and tw % seg == 0 and 8 % (tw // seg) == 0
        assert th == (8 // (tw // seg)) * (128 // seg)


def test_correlated_inputs_have_the_token_similarity_of_the_paper():
    """Appx A.1: tensors of consecutive tokens are about 0.87 similar; the i.i.d. recipe gives about 0."""
    L, H, D, n = 2, 8, 128, 256
    x = kv_synth.make_kv_correlated(L, H, D, n, torch.float32, seed=11).reshape(L, 2, n, H * D).double()
    y = kv_synth.make_kv(L, H, D, n, torch.float32, seed=11).reshape(L, 2, n, H * D).double()

    def token_similarity(v):
        # correlation over channels between token t and t+1, values taken relative to their channel scale
        v = v / v.std(dim=2, keepdim=True)
        a, b = v[:, :, :-1], v[:, :, 1:]
        a = a - a.mean(dim=-1, keepdim=True)
        b = b - b.mean(dim=-1, keepdim=True)
        return float(((a * b).sum(-1) / (a.norm(dim=-1) * b.norm(dim=-1))).mean())

    assert 0.80 < token_similarity(x) < 0.93
    assert abs(token_similarity(y)) < 0.05
    # seeded: the same call gives the same tensor
    assert torch.equal(kv_synth.make_kv_correlated(1, 2, 16, 8, torch.float16, seed=3),
                       kv_synth.make_kv_correlated(1, 2, 16, 8, torch.float16, seed=3))
