"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these tests calls the oracle to produce its own expected value: expected
values come from the paper's worked tiles (tests/golden/tile_examples.txt),
numpy / torch library routines on special cases, exact rational arithmetic,
brute force on tiny shapes and invariants of a uniform quantizer.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest
import torch

import kv_synth

HERE = os.path.dirname(os.path.abspath(__file__))

F16, BF16 = 0, 1


def small_layout(o, **kw):
    base = dict(L=4, H=2, D=16, dtype=F16, T=24, th=4, tw=8, TX=2, TY=3, k_mode=0, v_mode=1)
    base.update(kw)
    return o.make_layout(**base)


def rand_kv(lo, n_tokens, seed=0):
    dt = torch.float16 if lo.dtype == F16 else torch.bfloat16
    return kv_synth.make_kv(lo.L, lo.H, lo.D, n_tokens, dt, seed)


# ------------------------------------------------------------------ conversions


def test_widen_f16_all_patterns_match_numpy(oracle):
    bits = np.arange(65536, dtype=np.uint16)
    want = bits.view(np.float16).astype(np.float32)
    got = np.array([oracle.widen(int(b), F16) for b in bits], dtype=np.float32)
    finite = np.isfinite(want)
    assert np.array_equal(got[finite].view(np.uint32), want[finite].view(np.uint32))
    assert np.array_equal(np.isnan(got), np.isnan(want))
    assert np.array_equal(got[np.isinf(want)], want[np.isinf(want)])


def test_widen_bf16_matches_torch(oracle):
    bits = np.arange(0, 65536, 7, dtype=np.uint16)
    want = torch.from_numpy(bits.view(np.int16)).view(torch.bfloat16).to(torch.float32).numpy()
    got = np.array([oracle.widen(int(b), BF16) for b in bits], dtype=np.float32)
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok].view(np.uint32), want[ok].view(np.uint32))


def _narrow_cases():
    rng = np.random.default_rng(1)
    xs = [rng.standard_normal(4000).astype(np.float32) * s for s in (1e-8, 1e-5, 1e-3, 1.0, 50.0, 3e4, 7e4)]
    # exact ties between neighbouring fp16 values (and bf16 values), both parities
    h = rng.integers(0, 0x7BFF, 3000).astype(np.uint16)
    lo16 = h.view(np.float16).astype(np.float32)
    hi16 = (h + 1).astype(np.uint16).view(np.float16).astype(np.float32)
    xs.append((lo16 + hi16) / 2)  # exact in fp32: 11+1 significant bits
    b = rng.integers(0x0001, 0x7F7F, 3000).astype(np.uint32)
    tie_b = ((b << 16) | 0x8000).astype(np.uint32).view(np.float32)
    xs.append(tie_b)
    xs.append(np.array([0.0, -0.0, 65504.0, 65519.9, 65520.0, 65536.0, -65520.0, 2.0**-24, 2.0**-25, 1.5 * 2.0**-25,
                        2.0**-14, 2.0**-14 - 2.0**-25, 3.3895314e38, 1e-40, -1e-45], dtype=np.float32))
    x = np.concatenate(xs)
    return np.concatenate([x, -x])


def test_narrow_f16_matches_numpy(oracle):
    x = _narrow_cases()
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = np.array([oracle.narrow(v, F16) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


def test_narrow_bf16_matches_torch(oracle):
    x = _narrow_cases()
    want = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = np.array([oracle.narrow(v, BF16) for v in x], dtype=np.uint16)
    assert np.array_equal(got, want)


# ------------------------------------------------------------------ index map


def test_tile_examples_from_paper(oracle):
    """Sec. 3.2.2 closing paragraph + rules i-iii, hand-evaluated fixture."""
    rows = [ln.split() for ln in open(os.path.join(HERE, "golden", "tile_examples.txt")) if ln.strip() and ln[0] != "#"]
    assert len(rows) >= 16
    for H, D, th, tw, h, d, row, col in (map(int, r) for r in rows):
        lo = oracle.make_layout(L=3, H=H, D=D, dtype=F16, T=4, th=th, tw=tw, TX=2, TY=2)
        W = lo.TX * tw
        # token 0 sits at tile position (0, 0) of frame 0, layer 0 is plane 0
        off = oracle.frame_offset(lo, 0, 0, 0, h, d)
        assert divmod(off, W) == (row, col), (H, D, th, tw, h, d)


@pytest.mark.parametrize("H,D,th,tw", [(32, 128, 8, 512), (8, 128, 8, 128), (8, 128, 16, 64), (4, 16, 1, 64), (4, 16, 64, 1)])
def test_tile_is_row_major_reshape(oracle, H, D, th, tw):
    """The tile is numpy's reshape of the H*D vector (Sec. 3.2.2: 'reshaped')."""
    lo = oracle.make_layout(L=1, H=H, D=D, dtype=F16, T=1, th=th, tw=tw, TX=1, TY=1)
    tile = np.arange(H * D).reshape(H, D).reshape(th, tw)  # heads in order, in-head order kept
    got = np.empty((th, tw), dtype=np.int64)
    for h in range(H):
        for d in range(0, D, max(1, D // 8)):
            r, c = divmod(oracle.frame_offset(lo, 0, 0, 0, h, d), tw)
            got[r, c] = h * D + d
            assert tile[r, c] == h * D + d


@pytest.mark.parametrize("H,D,h1,d1", [(32, 128, 8, 1), (32, 128, 8, 4), (8, 128, 4, 2), (8, 128, 8, 2), (8, 128, 1, 16),
                                       (4, 16, 2, 2), (4, 16, 1, 1), (4, 16, 4, 16)])
def test_two_level_tile_is_numpy_reshape_transpose_reshape(oracle, H, D, h1, d1):
    """Sec. 3.2.2: head_num -> (h1, h2), head_dim -> (d1, d2), tile (h1*d1, h2*d2) -- e.g. (32,128) -> (8,4) x
    (1,128) -> (8,512).  As numpy states it: the [h1][h2][d1][d2] view of the token's [H][D] matrix with the two
    middle axes exchanged, flattened to two axes.  No element leaves its head (rule i), runs of d2 elements keep their
    order (rule ii), heads keep theirs (rule iii)."""
    h2, d2 = H // h1, D // d1
    th, tw = h1 * d1, h2 * d2
    lo = oracle.make_layout(L=1, H=H, D=D, dtype=F16, T=1, th=th, tw=tw, TX=1, TY=1, seg=d2)
    assert oracle.lib().kvco_check(lo) == 0
    tile = np.arange(H * D).reshape(h1, h2, d1, d2).transpose(0, 2, 1, 3).reshape(th, tw)
    for h in range(H):
        for d in range(D):
            r, c = divmod(oracle.frame_offset(lo, 0, 0, 0, h, d), tw)
            assert tile[r, c] == h * D + d, (h, d)
    if d1 == 1 or h2 == 1:   # these members of the family are the plain row-major retile: seg = 0 means the same
        lo0 = oracle.make_layout(L=1, H=H, D=D, dtype=F16, T=1, th=th, tw=tw, TX=1, TY=1)
        assert all(oracle.frame_offset(lo0, 0, 0, 0, h, d) == oracle.frame_offset(lo, 0, 0, 0, h, d)
                   for h in range(H) for d in range(0, D, 3))


def test_two_level_tile_rejects_inconsistent_segments(oracle):
    ok = dict(L=1, H=8, D=128, dtype=F16, T=1, TX=1, TY=1)
    check = oracle.lib().kvco_check
    assert check(oracle.make_layout(th=8, tw=128, seg=64, **ok)) == 0    # heads (4,2), dims (2,64)
    assert check(oracle.make_layout(th=16, tw=64, seg=16, **ok)) == 0    # heads (2,4), dims (8,16)
    assert check(oracle.make_layout(th=8, tw=128, seg=48, **ok)) != 0    # 48 divides neither 128
    assert check(oracle.make_layout(th=8, tw=128, seg=256, **ok)) != 0   # longer than a head
    assert check(oracle.make_layout(th=1, tw=1024, seg=64, **ok)) != 0   # a row would need 16 heads, there are 8


def test_rules_order_preserving(oracle):
    """Rules i-iii: raster order of a token's bytes == (head, dim) order."""
    lo = oracle.make_layout(L=1, H=8, D=32, dtype=F16, T=1, th=16, tw=16, TX=1, TY=1)
    offs = [oracle.frame_offset(lo, 0, 0, 0, h, d) for h in range(8) for d in range(32)]
    assert offs == sorted(offs) and len(set(offs)) == len(offs)


def test_temporal_alignment_and_groups(oracle):
    """Sec. 3.2.1 steps 2-3: the F tokens of a group share (plane, y, x) in F
    consecutive frames; the next group starts a new tile position in the first frame."""
    lo = small_layout(oracle)
    F = oracle.frames_per_group(lo)
    assert F == 4  # ceil(24 / 6)
    plane = lo.TY * lo.th * lo.TX * lo.tw
    frame = 3 * plane
    for kind, l, h, d in itertools.product((0, 1), range(lo.L), range(lo.H), (0, 5, 15)):
        for t in range(lo.T - 1):
            a = oracle.frame_offset(lo, kind, l, t, h, d)
            b = oracle.frame_offset(lo, kind, l, t + 1, h, d)
            if (t + 1) % F != 0:
                assert b - a == frame  # same pixel, next frame
            else:
                assert (a // frame) % F == F - 1 and (b // frame) % F == 0
                assert b % frame != a % frame  # a different tile position


def test_tile_positions_raster_order(oracle):
    """F = 1, tile (1, C): a plane viewed as [TY][TX][C] lists tokens in raster order."""
    lo = oracle.make_layout(L=3, H=2, D=8, dtype=F16, T=12, th=1, tw=16, TX=3, TY=4)
    assert oracle.frames_per_group(lo) == 1
    idx = np.arange(12 * 16).reshape(4, 3, 16)  # [ty][tx][channel] -> token*16 + channel
    flat = idx.reshape(4, 3 * 16).reshape(-1)  # the plane as [Hp=4][W=48] row-major
    for t in range(12):
        for e in (0, 7, 15):
            assert flat[oracle.frame_offset(lo, 0, 0, t, e // 8, e % 8)] == t * 16 + e


def test_three_layers_three_planes(oracle):
    """Sec. 3.2.1 step 1 / last sentence: layers 3g, 3g+1, 3g+2 are the planes of one frame."""
    lo = small_layout(oracle, L=7)
    F = oracle.frames_per_group(lo)
    plane = lo.TY * lo.th * lo.TX * lo.tw
    LG = 3
    assert oracle.frame_bytes(lo) == 2 * LG * F * 3 * plane
    for kind, l, t in itertools.product((0, 1), range(7), (0, 1, 9, 23)):
        off = oracle.frame_offset(lo, kind, l, t, 1, 3)
        frame_idx, rest = divmod(off, 3 * plane)
        assert rest // plane == l % 3
        assert frame_idx == (kind * LG + l // 3) * F + t % F
        # the three layers of a group differ only in the plane
        if l % 3 == 0 and l + 2 < 7:
            o1 = oracle.frame_offset(lo, kind, l + 1, t, 1, 3)
            o2 = oracle.frame_offset(lo, kind, l + 2, t, 1, 3)
            assert (o1 - off, o2 - off) == (plane, 2 * plane)


@pytest.mark.parametrize("kw", [dict(), dict(L=3, T=7, TX=1, TY=2), dict(L=1, H=1, D=8, th=1, tw=8, T=5, TX=2, TY=2),
                                dict(L=5, th=32, tw=1, T=6, TX=3, TY=1),
                                dict(L=2, H=4, D=16, th=4, tw=16, seg=8, T=5, TX=2, TY=2)])
def test_bijection_brute_force(oracle, kw):
    """Every valid element has its own byte inside the chunk section; count = 2*L*T*C."""
    lo = small_layout(oracle, **kw)
    seen = set()
    for kind, l, t, h, d in itertools.product((0, 1), range(lo.L), range(lo.T), range(lo.H), range(lo.D)):
        off = oracle.frame_offset(lo, kind, l, t, h, d)
        assert 0 <= off < oracle.frame_bytes(lo)
        seen.add(off)
    assert len(seen) == 2 * lo.L * lo.T * lo.H * lo.D


def test_meta_offsets_disjoint_and_sized(oracle):
    for km, vm in itertools.product((0, 1), (0, 1)):
        lo = small_layout(oracle, k_mode=km, v_mode=vm)
        seen = set()
        for kind, l, t, h, d in itertools.product((0, 1), range(lo.L), range(lo.T), range(lo.H), range(lo.D)):
            seen.add(oracle.meta_offset(lo, kind, l, t, h, d))
        n_pairs = sum(lo.L * lo.H * lo.D if m == 0 else lo.L * lo.T * lo.H for m in (km, vm))
        assert len(seen) == n_pairs and max(seen) + 2 == 2 * n_pairs == oracle.meta_floats(lo)
        assert all(o % 2 == 0 for o in seen)


def test_sizes_of_default_geometry(oracle):
    """Sizes used by the benchmark configurations (8 KV heads x 128, T = 2048, F = 4)."""
    lo = oracle.make_layout(L=32, H=8, D=128, dtype=F16, T=2048, th=8, tw=128, TX=8, TY=64)
    assert oracle.frames_per_group(lo) == 4
    assert oracle.frame_bytes(lo) == 2 * 11 * 4 * 3 * 512 * 1024 == 138_412_032
    assert oracle.meta_floats(lo) * 4 == 32 * 1024 * 8 + 32 * 2048 * 8 * 8 == 4_456_448


# ------------------------------------------------------------------ pack: layout of real data


def test_pack_special_case_is_numpy_reshape(oracle):
    """L = 3, F = 1, tile (1, C), per-channel groups: plane pl of the K frame is the
    [T][C] code matrix of layer pl, computed here with numpy alone."""
    T, H, D = 40, 2, 8
    C = H * D
    lo = oracle.make_layout(L=3, H=H, D=D, dtype=F16, T=T, th=1, tw=C, TX=1, TY=T, k_mode=0, v_mode=0)
    kv = rand_kv(lo, T, seed=3)
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), T)
    x = kv.to(torch.float32).numpy().reshape(3, 2, T, C)
    fr = frames.reshape(2, 1, 1, 3, T, C)
    me = meta.reshape(2, 3, C, 2)
    for kind in (0, 1):
        for l in range(3):
            a = x[l, kind]
            mn, mx = a.min(0), a.max(0)
            rng = (mx - mn).astype(np.float32)
            inv = np.float32(255.0) / rng
            codes = np.clip(np.rint(((a - mn).astype(np.float32) * inv).astype(np.float32)), 0, 255).astype(np.uint8)
            assert np.array_equal(fr[kind, 0, 0, l], codes)
            assert np.array_equal(me[kind, l, :, 1], mn)
            assert np.array_equal(me[kind, l, :, 0], rng / np.float32(255.0))


def test_pack_per_token_special_case_numpy(oracle):
    """Same special case with per-(token, head) groups for both kinds."""
    T, H, D = 12, 3, 8
    C = H * D
    lo = oracle.make_layout(L=3, H=H, D=D, dtype=BF16, T=T, th=1, tw=C, TX=1, TY=T, k_mode=1, v_mode=1)
    kv = rand_kv(lo, T, seed=4)
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), T)
    x = kv.to(torch.float32).numpy().reshape(3, 2, T, H, D)
    fr = frames.reshape(2, 1, 1, 3, T, H, D)
    me = meta.reshape(2, 3, T, H, 2)
    for kind in (0, 1):
        for l in range(3):
            a = x[l, kind]
            mn, mx = a.min(-1, keepdims=True), a.max(-1, keepdims=True)
            rng = (mx - mn).astype(np.float32)
            inv = np.float32(255.0) / rng
            codes = np.clip(np.rint(((a - mn).astype(np.float32) * inv).astype(np.float32)), 0, 255).astype(np.uint8)
            assert np.array_equal(fr[kind, 0, 0, l], codes)
            assert np.array_equal(me[kind, l, :, :, 1], mn[..., 0])


def test_pack_zero_fill_short_chunk_and_pad_planes(oracle):
    """Bytes of absent tokens, unused tile positions and planes of layers >= L are 0;
    per-token pairs of absent tokens are {0, 0}; every other byte belongs to one element."""
    lo = small_layout(oracle, L=4, T=22)  # G = 6, F = 4: positions for 24 tokens, 22 used
    n_tokens = 22 + 9  # second chunk holds 9 tokens
    kv = rand_kv(lo, n_tokens, seed=5)
    # make sure real codes are rarely 0 in what we count below: irrelevant, we mask by position
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), n_tokens)
    fb, mf = oracle.frame_bytes(lo), oracle.meta_floats(lo)
    assert frames.size == 2 * fb and meta.size == 2 * mf
    for c, n in ((0, 22), (1, 9)):
        valid = np.zeros(fb, dtype=bool)
        for kind, l, t, h, d in itertools.product((0, 1), range(lo.L), range(n), range(lo.H), range(lo.D)):
            valid[oracle.frame_offset(lo, kind, l, t, h, d)] = True
        sec = frames[c * fb:(c + 1) * fb]
        assert valid.sum() == 2 * lo.L * n * lo.H * lo.D
        assert not sec[~valid].any()
        # V block is per token: pairs of tokens >= n are zero
        vm = meta[c * mf + oracle.meta_kind_offset(lo, 1):(c + 1) * mf].reshape(lo.L, lo.T, lo.H, 2)
        assert not vm[:, n:].any()
        assert np.isfinite(meta[c * mf:(c + 1) * mf]).all()


def test_pack_respects_strides(oracle):
    lo = small_layout(oracle, L=3)
    n = 30
    C = lo.H * lo.D
    kv = rand_kv(lo, n, seed=6)
    dense = kv_synth.to_u16(kv)
    # embed in a larger buffer: token stride 2C, gaps between kinds and layers
    ts, ks = 2 * C, n * 2 * C + 16
    ls = 2 * ks + 8
    big = np.full(lo.L * ls, 0x7C00, dtype=np.uint16)  # +inf everywhere else: must never be read
    d5 = dense.reshape(lo.L, 2, n, C)
    for l in range(lo.L):
        for k in (0, 1):
            for t in range(n):
                big[l * ls + k * ks + t * ts: l * ls + k * ks + t * ts + C] = d5[l, k, t]
    f1, m1 = oracle.pack(lo, dense.reshape(-1), n)
    f2, m2 = oracle.pack(lo, big, n, strides=(ls, ks, ts))
    assert np.array_equal(f1, f2) and np.array_equal(m1.view(np.uint32), m2.view(np.uint32))
    out = np.full(lo.L * ls, 0xFFFF, dtype=np.uint16)
    oracle.restore(lo, f2, m2, n, out=out, strides=(ls, ks, ts))
    ref = oracle.restore(lo, f1, m1, n).reshape(lo.L, 2, n, C)
    touched = np.zeros(out.size, dtype=bool)
    for l in range(lo.L):
        for k in (0, 1):
            for t in range(n):
                s = l * ls + k * ks + t * ts
                assert np.array_equal(out[s:s + C], ref[l, k, t])
                touched[s:s + C] = True
    assert (out[~touched] == 0xFFFF).all()


# ------------------------------------------------------------------ quantizer invariants


@pytest.mark.parametrize("dtype", [F16, BF16])
@pytest.mark.parametrize("modes", [(0, 1), (1, 0)])
def test_round_trip_error_bound(oracle, dtype, modes):
    """Uniform quantizer: |x - x_hat| <= scale/2 up to the fp32 rounding of the
    position (x - mn) * inv and of scale: each of the subtraction, inv, their
    product and scale carries a relative error <= 2^-24 on a position <= 255, so
    the slack is 4 * 255 * 2^-24 < 2^-14 steps.  The stored 16-bit value is the
    nearest to x_hat."""
    lo = small_layout(oracle, dtype=dtype, k_mode=modes[0], v_mode=modes[1], L=3)
    n = 24 + 11
    kv = rand_kv(lo, n, seed=7)
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), n)
    out = oracle.restore(lo, frames, meta, n).reshape(lo.L, 2, n, lo.H, lo.D)
    tdt = torch.float16 if dtype == F16 else torch.bfloat16
    outf = torch.from_numpy(out.view(np.int16)).view(tdt).to(torch.float64).numpy()
    x = kv.to(torch.float64).numpy()
    fb, mf = oracle.frame_bytes(lo), oracle.meta_floats(lo)
    ulp_rel = 2.0 ** -11 if dtype == F16 else 2.0 ** -8
    worst = 0.0
    for l, kind, p, h, d in itertools.product(range(lo.L), (0, 1), range(n), range(lo.H), range(lo.D)):
        c, t = divmod(p, lo.T)
        code = int(frames[c * fb + oracle.frame_offset(lo, kind, l, t, h, d)])
        mo = c * mf + oracle.meta_offset(lo, kind, l, t, h, d)
        scale, mn = float(meta[mo]), float(meta[mo + 1])
        xh = code * scale + mn  # exact enough in fp64: 8-bit x 24-bit product
        err = abs(x[l, kind, p, h, d] - xh)
        assert err <= scale * (0.5 + 2.0 ** -14) + 1e-30, (l, kind, p, h, d, code, scale, mn)
        worst = max(worst, err / scale if scale else 0.0)
        o = outf[l, kind, p, h, d]
        assert abs(o - xh) <= abs(xh) * ulp_rel * (1 + 2.0 ** -20) + 2.0 ** -25
    assert worst > 0.45  # the bound is reached: the quantizer is not trivially exact


def test_group_params_extremes_and_meta(oracle):
    rng = np.random.default_rng(11)
    for _ in range(200):
        n = int(rng.integers(2, 70))
        xs = (rng.standard_normal(n) * 10.0 ** rng.uniform(-3, 3)).astype(np.float16).astype(np.float32)
        scale, mn, inv = oracle.group_params(xs)
        assert mn.view(np.uint32) == (xs.min() + np.float32(0)).view(np.uint32)  # an input value, bit for bit
        rngf = float(xs.max()) - float(xs.min())  # exact in fp64
        if rngf == 0:
            assert scale == 0 and inv == 0
            continue
        assert abs(float(scale) * 255 - rngf) <= 2.0 ** -22 * rngf
        assert abs(float(inv) * rngf - 255) <= 2.0 ** -21 * 255
        # element equal to the minimum -> code 0 and exact restore; maximum -> 255
        assert oracle.quantize(xs.min(), mn, inv) == 0
        assert oracle.quantize(xs.max(), mn, inv) == 255
        assert oracle.dequantize(0, scale, mn) == mn
        # monotone codes
        order = np.argsort(xs)
        codes = [oracle.quantize(v, mn, inv) for v in xs[order]]
        assert codes == sorted(codes)


def test_division_and_fma_are_correctly_rounded(oracle):
    """scale, inv and the dequantized value against exact rational arithmetic."""
    rng = np.random.default_rng(12)

    def nearest_f32(fr):  # candidates around float(fr)
        c = np.float32(float(fr))
        cands = [c, np.nextafter(c, np.float32(np.inf)), np.nextafter(c, np.float32(-np.inf))]
        return min(abs(Fraction(float(v)) - fr) for v in cands)

    for _ in range(300):
        xs = (rng.standard_normal(5) * 10.0 ** rng.uniform(-4, 4)).astype(np.float32)
        scale, mn, inv = oracle.group_params(xs)
        r = Fraction(float(np.float32(xs.max() - mn)))
        assert abs(Fraction(float(scale)) - r / 255) == nearest_f32(r / 255)
        assert abs(Fraction(float(inv)) - 255 / r) == nearest_f32(255 / r)
        code = int(rng.integers(0, 256))
        exact = code * Fraction(float(scale)) + Fraction(float(mn))
        got = oracle.dequantize(code, scale, mn)
        assert abs(Fraction(float(got)) - exact) == nearest_f32(exact)


def test_rounding_is_half_to_even_and_clamped(oracle):
    # mn = 0, inv = 1: positions k + 0.5 are exact ties
    assert [oracle.quantize(v, 0.0, 1.0) for v in (0.5, 1.5, 2.5, 3.5, 254.5, 255.4, 300.0, -3.0)] == \
        [0, 2, 2, 4, 254, 255, 255, 0]


def test_constant_group_and_negative_zero(oracle):
    scale, mn, inv = oracle.group_params(np.array([-0.0, -0.0, -0.0], dtype=np.float32))
    assert scale == 0 and inv == 0 and mn.view(np.uint32) == 0  # +0.0
    scale, mn, inv = oracle.group_params(np.array([3.25] * 9, dtype=np.float32))
    assert (scale, mn, inv) == (0, 3.25, 0)
    assert oracle.quantize(3.25, mn, inv) == 0 and oracle.dequantize(0, scale, mn) == np.float32(3.25)
    lo = small_layout(oracle, L=1, T=6, TX=1, TY=2)
    kv = torch.full((1, 2, 6, lo.H, lo.D), -1.5, dtype=torch.float16)
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), 6)
    assert not frames.any()
    out = oracle.restore(lo, frames, meta, 6)
    assert np.array_equal(out, kv_synth.to_u16(kv).reshape(-1))


def test_per_channel_stats_use_valid_tokens_only(oracle):
    """A short last chunk: groups span that chunk's tokens only, each chunk has its own groups."""
    lo = small_layout(oracle, L=1, k_mode=0, v_mode=0)
    n = lo.T + 5
    kv = rand_kv(lo, n, seed=8)
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), n)
    x = kv.to(torch.float32).numpy().reshape(1, 2, n, lo.H * lo.D)
    mf = oracle.meta_floats(lo)
    for c, (a, b) in enumerate(((0, lo.T), (lo.T, n))):
        me = meta[c * mf:(c + 1) * mf].reshape(2, lo.H * lo.D, 2)
        for kind in (0, 1):
            assert np.array_equal(me[kind, :, 1], x[0, kind, a:b].min(0) + np.float32(0))


# ------------------------------------------------------------------ restore placement


def test_paged_identity_table_equals_contiguous(oracle):
    lo = small_layout(oracle, L=3)
    n = lo.T * 2 + 7
    bs = 4
    nb = (n + bs - 1) // bs
    kv = rand_kv(lo, n, seed=9)
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), n)
    C = lo.H * lo.D
    contiguous = oracle.restore(lo, frames, meta, n).reshape(lo.L, 2, n, C)
    caches = [np.full(2 * nb * bs * C, 0xDEAD, dtype=np.uint16) for _ in range(lo.L)]
    err = oracle.restore_paged(lo, frames, meta, 0, n, caches, nb, bs, np.arange(nb))
    assert err == 0
    for l in range(lo.L):
        got = caches[l].reshape(2, nb * bs, C)
        assert np.array_equal(got[:, :n], contiguous[l])
        assert (got[:, n:] == 0xDEAD).all()  # slots past the last token untouched


def test_paged_permutation_poison_and_bad_ids(oracle):
    lo = small_layout(oracle, L=2)
    n = lo.T * 2  # two chunks; restore them in two calls via first_token
    bs, nb = 8, 11  # 6 logical blocks in an 11-block cache
    nl = n // bs
    C = lo.H * lo.D
    kv = rand_kv(lo, n, seed=10)
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), n)
    contiguous = oracle.restore(lo, frames, meta, n).reshape(lo.L, 2, nl, bs, C)
    table = kv_synth.make_block_table(nl, nb, seed=1).numpy().copy()
    table[4] = nb + 3   # out of range (high)
    table[1] = -1       # out of range (negative)
    caches = [np.full(2 * nb * bs * C, 0xDEAD, dtype=np.uint16) for _ in range(lo.L)]
    fb, mf = oracle.frame_bytes(lo), oracle.meta_floats(lo)
    e0 = oracle.restore_paged(lo, frames[:fb], meta[:mf], 0, lo.T, caches, nb, bs, table)
    e1 = oracle.restore_paged(lo, frames[fb:], meta[mf:], lo.T, lo.T, caches, nb, bs, table)
    assert (e0 | e1) == 1
    used = {int(p): b for b, p in enumerate(table) if 0 <= p < nb}
    for l in range(lo.L):
        got = caches[l].reshape(2, nb, bs, C)
        for phys in range(nb):
            if phys in used:
                assert np.array_equal(got[:, phys], contiguous[l][:, used[phys]])
            else:
                assert (got[:, phys] == 0xDEAD).all()


def test_oracle_rejects_bad_arguments(oracle):
    lo = small_layout(oracle)
    bad = small_layout(oracle, th=5)
    kv = kv_synth.to_u16(rand_kv(lo, 4)).reshape(-1)
    with pytest.raises(ValueError):
        oracle.pack(bad, kv, 4)
    frames, meta = oracle.pack(lo, kv, 4)
    caches = [np.zeros(2 * 2 * 4 * lo.H * lo.D, dtype=np.uint16) for _ in range(lo.L)]
    with pytest.raises(ValueError):  # first_token not a multiple of T
        oracle.restore_paged(lo, frames, meta, 3, 4, caches, 2, 4, np.arange(2))
    with pytest.raises(ValueError):  # table too short: 1 block of 4 slots for 5 tokens
        oracle.restore_paged(lo, frames, meta, 0, 5, caches, 2, 4, np.arange(1))


# ------------------------------------------------------------------ frame-wise restoration


def test_frame_restore_writes_exactly_its_tokens_and_layers(oracle):
    """Sec. 3.3.2 + Sec. 3.2.1 step 3: one frame (kind, lg, f) carries the tokens t % F == f of layers 3lg..3lg+2;
    everything else in the cache stays poison, and the written values are those of the chunk-level restore."""
    lo = small_layout(oracle, L=5, T=22)  # LG = 2 (second group has 2 layers), F = 4, short second chunk
    n = 22 + 9
    bs, nb = 4, 11
    C = lo.H * lo.D
    F = oracle.frames_per_group(lo)
    kv = rand_kv(lo, n, seed=21)
    frames, meta = oracle.pack(lo, kv_synth.to_u16(kv), n)
    fb, mf, fs = oracle.frame_bytes(lo), oracle.meta_floats(lo), oracle.frame_size(lo)
    assert fb == 2 * 2 * F * fs
    table = kv_synth.make_block_table((n + bs - 1) // bs, nb, seed=2).numpy()
    whole = [np.full(2 * nb * bs * C, 0xDEAD, dtype=np.uint16) for _ in range(lo.L)]
    oracle.restore_paged(lo, frames, meta, 0, n, whole, nb, bs, table)
    union = [np.full(2 * nb * bs * C, 0xDEAD, dtype=np.uint16) for _ in range(lo.L)]
    for c, nt in ((0, 22), (1, 9)):
        for kind, lg, f in itertools.product((0, 1), (0, 1), range(F)):
            start = oracle.frame_start(lo, kind, lg, f)
            assert start == ((kind * 2 + lg) * F + f) * fs  # frames are laid out [kind][lg][f]
            frame = frames[c * fb + start: c * fb + start + fs]
            one = [np.full(2 * nb * bs * C, 0xDEAD, dtype=np.uint16) for _ in range(lo.L)]
            err = oracle.restore_paged_frame(lo, frame, meta[c * mf:(c + 1) * mf], kind, lg, f, c * lo.T, nt, one, nb, bs, table)
            assert err == 0
            oracle.restore_paged_frame(lo, frame, meta[c * mf:(c + 1) * mf], kind, lg, f, c * lo.T, nt, union, nb, bs, table)
            for l in range(lo.L):
                got = one[l].reshape(2, nb, bs, C)
                ref = whole[l].reshape(2, nb, bs, C)
                for k2 in (0, 1):
                    for p in range(nb * bs):
                        blk, slot = divmod(p, bs)
                        # which sequence position lives here?
                        logical = np.flatnonzero(table == blk)
                        pos = logical[0] * bs + slot if logical.size else -1
                        t = pos - c * lo.T
                        mine = (k2 == kind and l // 3 == lg and 0 <= t < nt and t % F == f and pos >= 0)
                        if mine:
                            assert np.array_equal(got[k2, blk, slot], ref[k2, blk, slot])
                            assert (got[k2, blk, slot] != 0xDEAD).any()
                        else:
                            assert (got[k2, blk, slot] == 0xDEAD).all()
    for l in range(lo.L):  # all frames together == the chunk-level restore
        assert np.array_equal(union[l], whole[l])


def test_frame_restore_rejects_bad_arguments(oracle):
    lo = small_layout(oracle)
    kv = kv_synth.to_u16(rand_kv(lo, 8)).reshape(-1)
    frames, meta = oracle.pack(lo, kv, 8)
    fs = oracle.frame_size(lo)
    caches = [np.zeros(2 * 2 * 4 * lo.H * lo.D, dtype=np.uint16) for _ in range(lo.L)]
    for kind, lg, f in ((2, 0, 0), (0, 2, 0), (0, 0, 4), (0, -1, 0)):
        with pytest.raises(ValueError):
            oracle.restore_paged_frame(lo, frames[:fs], meta, kind, lg, f, 0, 8, caches, 2, 4, np.arange(2))


# ------------------------------------------------------------------ Appx A.3 admission condition


def test_admission_uniform_times_closed_form():
    """Uniform stage times d (fetch) and c (compute), 0 < d < c: stage k violates k*d <= (k-1)*c iff k < c/(c-d),
    so the stages that must be buffered first are 1 .. ceil(c/(c-d)) - 1 (all n when that exceeds n)."""
    from oracle import admission
    for d, c, n in [(1, 2, 8), (3, 4, 8), (5, 7, 8), (3, 4, 2), (9, 10, 32), (1, 100, 5)]:
        want = min(n, -(-c // (c - d)) - 1)
        assert admission.min_buffered([d] * n, [c] * n) == want, (d, c, n)
        for b in range(n + 1):
            assert admission.condition_holds([d] * n, [c] * n, b) == (b >= want)
    # fetch never faster than compute: nothing can be hidden; free fetch: nothing to hide
    assert admission.min_buffered([2.0] * 6, [2.0] * 6) == 6
    assert admission.min_buffered([3.0] * 6, [2.0] * 6) == 6
    assert admission.min_buffered([0.0] * 6, [2.0] * 6) == 0
    assert admission.min_buffered([0.0] * 6, [0.0] * 6) == 0  # 0 <= 0 holds: the bound is not strict


def test_admission_hand_evaluated_example():
    """Four stages, checked by hand: prefix sums of fetch 2,3,4,5 against shifted prefix sums of compute 0,4,5,6."""
    from oracle import admission
    f, c = [2, 1, 1, 1], [4, 1, 1, 9]
    assert not admission.condition_holds(f, c, 0)      # k = 1: 2 <= 0 fails
    assert admission.condition_holds(f, c, 1)          # k = 2..4: 3 <= 4, 4 <= 5, 5 <= 6
    assert admission.min_buffered(f, c) == 1
    f2 = [2, 1, 1, 3]                                   # k = 4: 7 <= 6 fails
    assert not admission.condition_holds(f2, c, 3) and admission.condition_holds(f2, c, 4)
    assert admission.min_buffered(f2, c) == 4
    # the compute time of the last stage never enters: nothing is fetched behind it
    assert admission.min_buffered(f, [4, 1, 1, 0]) == 1


def test_admission_monotone_and_empty_constraint_set():
    from oracle import admission
    rng = np.random.default_rng(5)
    for _ in range(200):
        n = int(rng.integers(1, 12))
        f, c = rng.uniform(0, 2, n).tolist(), rng.uniform(0, 3, n).tolist()
        holds = [admission.condition_holds(f, c, b) for b in range(n + 1)]
        assert holds[n]                                 # everything buffered: no inequality left
        assert holds == sorted(holds)                   # once it holds it keeps holding
        assert admission.min_buffered(f, c) == holds.index(True)


# ------------------------------------------------------------------ Alg. 1 adaptive-resolution selector


def load_alg1_tables():
    """{device: (sizes, latency rows by load, penalty)} from the tables the paper prints (Appx A.2)."""
    tables = {}
    for line in open(os.path.join(HERE, "golden", "alg1_lookup_tables.txt")):
        if line.startswith("#") or not line.strip():
            continue
        tok = line.split()
        dev = tables.setdefault(tok[0], {"load": {}, "penalty": None, "size": None})
        if tok[1] == "load":
            dev["load"][int(tok[2])] = [float(x) for x in tok[3:]]
        else:
            dev[tok[1]] = [float(x) for x in tok[2:]]
    out = {}
    for name, d in tables.items():
        rows = [d["load"][k] for k in range(1, len(d["load"]) + 1)]
        out[name] = (d["size"], rows, d["penalty"])
    return out


def load_alg1_cases():
    cases = []
    for line in open(os.path.join(HERE, "golden", "alg1_cases.txt")):
        if line.startswith("#") or not line.strip():
            continue
        dev, load, active, bw, chosen, bubble = line.split()
        cases.append((dev, int(load), int(active), float(bw), int(chosen), float(bubble)))
    return cases


def test_alg1_hand_evaluated_selections_on_the_papers_tables():
    from oracle import resolution
    tables = load_alg1_tables()
    assert set(tables) == {"H20", "L20", "A100"} and len(tables["H20"][1]) == 7
    cases = load_alg1_cases()
    assert len(cases) == 8
    for dev, load, active, bw, chosen, bubble in cases:
        sizes, rows, pen = tables[dev]
        r, b = resolution.select_resolution(sizes, rows, pen, load, active, bw)
        assert r == chosen, (dev, load, active, bw, r, b)
        assert abs(b - bubble) < 1e-8


def test_alg1_zero_bubble_ties_and_scaling():
    from oracle import resolution
    # a resolution whose transmission takes exactly as long as its decoding wins with bubble 0
    r, b = resolution.select_resolution([100, 200, 400], [[3.0, 2.0, 5.0]], [0, 0, 0], 1, -1, 100.0)
    assert (r, b) == (1, 0.0)
    # equal bubbles: the earlier resolution of the set is kept
    r, b = resolution.select_resolution([100, 300], [[2.0, 2.0]], [0, 0], 1, -1, 100.0)   # |1-2| = |3-2|
    assert (r, b) == (0, 1.0)
    # scaling every time by 4 (sizes x4 at the same bandwidth, latencies and penalties x4) changes no decision
    rng = np.random.default_rng(3)
    for _ in range(100):
        n, loads = int(rng.integers(1, 6)), int(rng.integers(1, 5))
        sizes = rng.uniform(50, 300, n)
        lat = rng.uniform(0.05, 0.6, (loads, n))
        pen = rng.uniform(0, 0.1, n)
        load, active, bw = int(rng.integers(1, loads + 1)), int(rng.integers(-1, n)), float(rng.uniform(100, 2000))
        r1, b1 = resolution.select_resolution(sizes, lat, pen, load, active, bw)
        r2, b2 = resolution.select_resolution(sizes * 4, lat * 4, pen * 4, load, active, bw)
        assert r1 == r2 and b2 == 4 * b1      # powers of two scale exactly in binary floating point
    assert resolution.est_bandwidth(256e6, 0.5) == 512e6
