"""CPU oracle of the codec-free proxy that ranks intra-frame tilings (Sec. 3.2.2).

TEST INFRASTRUCTURE ONLY: imported by tests/ alone.

The paper's search evaluates the size of the encoded video for every candidate tiling; that needs an H.265
encoder.  The proxy used here replaces the encoder by the first-order entropy of the residuals that a predictive
coder would have to store, for the predictors a video codec has: the pixel to the left and the pixel above
(intra prediction) and the same pixel of the previous frame (inter prediction; Sec. 3.2.1 step 3 puts consecutive
tokens there), the latter also after removing what its own left / upper neighbour already explains.  It is a
proxy, not the paper's objective: parity with the paper's compression ratios is unpinned.

Definitions (all arithmetic modulo 256 on the 8-bit codes of one plane sequence p[f][y][x], f = 0..F-1 the frames
of one (chunk, kind, layer), pixels outside the plane and frames before the first read as 0):
    L [f][y][x] = p[f][y][x] - p[f][y][x-1]                      every frame
    U [f][y][x] = p[f][y][x] - p[f][y-1][x]                      every frame
    T [f][y][x] = p[f][y][x] - p[f-1][y][x]                      frames f >= 1
    TL[f][y][x] = T[f][y][x] - T[f][y][x-1]                      frames f >= 1
    TU[f][y][x] = T[f][y][x] - T[f][y-1][x]                      frames f >= 1
Histogram k of a stream counts the values of residual k over the frames named.  Entropy of a histogram
H = -sum_i (n_i / N) log2(n_i / N) bits per pixel.  Cost of a stream in bits: the first frame of a group has no
frame to predict from, the others take the cheapest predictor:
    cost = Hp*W * min(H_L, H_U) + (F-1)*Hp*W * min(H_T, H_TL, H_TU)

Pins (tests marked "not gpu"): histograms of hand-made planes, entropy of a constant and of a uniform plane, a frame
repeated gives T = 0 everywhere, a plane constant along x (along y) gives L (U) = 0 off the border, total counts,
and invariance of T under any permutation of pixel positions (the temporal term cannot depend on the tile).
"""
import numpy as np

from . import kvco_py

N_RESIDUALS = 5
RES_L, RES_U, RES_T, RES_TL, RES_TU = range(5)


def plane_sequences(lo, frames, n_chunks):
    """View of `frames` (uint8, n_chunks chunk sections) as [chunk][kind][LG][F][3][Hp][W]."""
    F = kvco_py.frames_per_group(lo)
    LG = (lo.L + 2) // 3
    Hp, W = lo.TY * lo.th, lo.TX * lo.tw
    return np.asarray(frames, dtype=np.uint8).reshape(n_chunks, 2, LG, F, 3, Hp, W)


def _shift_x(a):
    out = np.zeros_like(a)
    out[..., 1:] = a[..., :-1]
    return out


def _shift_y(a):
    out = np.zeros_like(a)
    out[..., 1:, :] = a[..., :-1, :]
    return out


def stream_histograms(p):
    """p: uint8 [F][Hp][W], the frames of one (chunk, kind, layer).  Returns uint64 [5][256]."""
    p = np.asarray(p, dtype=np.uint8)
    hist = np.zeros((N_RESIDUALS, 256), dtype=np.uint64)
    res_l = p - _shift_x(p)          # uint8 arithmetic wraps modulo 256
    res_u = p - _shift_y(p)
    hist[RES_L] = np.bincount(res_l.reshape(-1), minlength=256)
    hist[RES_U] = np.bincount(res_u.reshape(-1), minlength=256)
    if p.shape[0] > 1:
        t = p[1:] - p[:-1]
        hist[RES_T] = np.bincount(t.reshape(-1), minlength=256)
        hist[RES_TL] = np.bincount((t - _shift_x(t)).reshape(-1), minlength=256)
        hist[RES_TU] = np.bincount((t - _shift_y(t)).reshape(-1), minlength=256)
    return hist


def residual_histograms(lo, frames, n_chunks):
    """Returns uint64 [n_chunks][2][L][5][256]; planes of layers >= L are not streams."""
    seq = plane_sequences(lo, frames, n_chunks)
    out = np.zeros((n_chunks, 2, lo.L, N_RESIDUALS, 256), dtype=np.uint64)
    for c in range(n_chunks):
        for kind in (0, 1):
            for l in range(lo.L):
                out[c, kind, l] = stream_histograms(seq[c, kind, l // 3, :, l % 3])
    return out


def entropy_bits_per_symbol(hist):
    h = np.asarray(hist, dtype=np.float64)
    n = h.sum()
    if n == 0:
        return 0.0
    q = h[h > 0] / n
    return float(-(q * np.log2(q)).sum())


def stream_cost_bits(lo, hist):
    """hist: [5][256] of one stream."""
    F = kvco_py.frames_per_group(lo)
    pixels = (lo.TY * lo.th) * (lo.TX * lo.tw)
    intra = min(entropy_bits_per_symbol(hist[RES_L]), entropy_bits_per_symbol(hist[RES_U]))
    cost = pixels * intra
    if F > 1:
        inter = min(entropy_bits_per_symbol(hist[k]) for k in (RES_T, RES_TL, RES_TU))
        cost += (F - 1) * pixels * inter
    return cost


def total_cost_bits(lo, hists):
    """hists: [n_chunks][2][L][5][256] -> sum of the stream costs, in bits."""
    h = np.asarray(hists).reshape(-1, N_RESIDUALS, 256)
    return float(sum(stream_cost_bits(lo, s) for s in h))


def tile_candidates(H, D, min_seg=8):
    """The tilings of Sec. 3.2.2 after rules i-iii: head_num = h1*h2, head_dim = d1*d2 (powers of two), tile
    (h1*d1, h2*d2).  Returns [(th, tw, seg)] with seg = d2 >= min_seg, in the order h1 ascending, d1 ascending."""
    out = []
    h1 = 1
    while h1 <= H:
        if H % h1 == 0:
            d1 = 1
            while d1 <= D:
                if D % d1 == 0 and D // d1 >= min_seg:
                    out.append((h1 * d1, (H // h1) * (D // d1), D // d1))
                d1 *= 2
        h1 *= 2
    return out
