"""Host-side behaviour of the C ABI that needs no GPU: the library loads, exports
every symbol the header declares, sizes agree with the oracle's, and every
host-checkable fault is rejected before anything could be enqueued."""
import ctypes
import os
import re

import numpy as np

import pytest

import paper_2602_09725_amd as kvc
from paper_2602_09725_amd import kvc as binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def good(**kw):
    base = dict(num_layers=32, num_kv_heads=8, head_dim=128, dtype=0, chunk_tokens=2048, tile_h=8, tile_w=128,
                tiles_x=8, tiles_y=64)
    base.update(kw)
    return kvc.Layout(**base)


def test_library_exports_every_declared_symbol(kvc_lib):
    header = open(os.path.join(ROOT, "include", "kvc.h")).read()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    names = set(re.findall(r"\b(kvc_[a-z_]+)\s*\(", body))
    assert {"kvc_pack", "kvc_restore", "kvc_restore_paged", "kvc_fetch_pipeline", "kvc_chunk_sizes",
            "kvc_restore_paged_frame", "kvc_restore_paged_frames", "kvc_fetch_pipeline_frames",
            "kvc_meta_staging_size", "kvc_admission_ok", "kvc_admission_min_buffered", "kvc_select_resolution",
            "kvc_est_bandwidth", "kvc_layout_set_resolution", "kvc_frame_size", "kvc_frame_offset",
            "kvc_layout_validate", "kvc_status_str", "kvc_blob_meta_offset"} <= names
    for n in names:
        assert hasattr(kvc_lib, n), f"libkvc.so does not export {n}"


def test_binding_struct_matches_header(kvc_lib):
    assert ctypes.sizeof(kvc.Layout) == 14 * 4
    assert kvc.layout_validate(good()) == 0
    lo = good()
    lo.struct_size = 48
    assert kvc.layout_validate(lo) == 1
    lo = good()
    lo.abi_version = 1
    assert kvc.layout_validate(lo) == 1


def test_chunk_sizes_agree_with_oracle(kvc_lib, oracle):
    for kw in (dict(), dict(num_layers=60, dtype=1), dict(num_layers=2), dict(k_mode=1, v_mode=0),
               dict(num_kv_heads=32, tile_h=8, tile_w=512, chunk_tokens=1000, tiles_x=3, tiles_y=7)):
        lo = good(**kw)
        fb, mb, F = kvc.chunk_sizes(lo)
        olo = oracle.make_layout(lo.num_layers, lo.num_kv_heads, lo.head_dim, lo.dtype, lo.chunk_tokens, lo.tile_h,
                                 lo.tile_w, lo.tiles_x, lo.tiles_y, lo.k_mode, lo.v_mode)
        assert (fb, mb, F) == (oracle.frame_bytes(olo), 4 * oracle.meta_floats(olo), oracle.frames_per_group(olo))
        assert kvc.blob_meta_offset(lo) == (fb + 255) // 256 * 256
    assert kvc.chunk_sizes(good())[:2] == (138_412_032, 4_456_448)


@pytest.mark.parametrize("kw", [dict(tile_w=100), dict(num_layers=0), dict(dtype=2), dict(k_mode=3), dict(tiles_x=0),
                                dict(chunk_tokens=-5), dict(tile_h=16), dict(tile_seg=-8), dict(tile_seg=48),
                                dict(tile_seg=256), dict(tile_h=1, tile_w=1024, tile_seg=64)])
def test_inconsistent_layouts_rejected(kvc_lib, kw):
    assert kvc.layout_validate(good(**kw)) == 1
    with pytest.raises(kvc.KvcError):
        kvc.chunk_sizes(good(**kw))


def test_two_level_tiles_validate_like_the_oracle(kvc_lib, oracle):
    """tile_seg = d2 of Sec. 3.2.2's two-level reshape: accepted exactly when the oracle accepts it; a run shorter than
    an 8-element atom is a valid layout the kernels do not cover."""
    for th, tw, seg in [(8, 128, 64), (16, 64, 16), (8, 128, 128), (8, 128, 0), (4, 256, 32), (8, 128, 48),
                        (8, 128, 256), (1, 1024, 64), (32, 32, 32), (64, 16, 16)]:
        lo = good(tile_h=th, tile_w=tw, tile_seg=seg)
        olo = oracle.make_layout(32, 8, 128, 0, 2048, th, tw, 8, 64, seg=seg)
        assert (kvc.layout_validate(lo) == 0) == (oracle.lib().kvco_check(olo) == 0), (th, tw, seg)
    lo = good(tile_h=128, tile_w=8, tile_seg=4)   # heads (4,2), dims (32,4)
    assert kvc.layout_validate(lo) == 0
    with pytest.raises(kvc.KvcError) as e:
        kvc.pack_plan(lo, (2 * 4096 * 1024, 4096 * 1024, 1024))
    assert e.value.status == 2


def test_data_calls_reject_bad_arguments_before_enqueueing(kvc_lib):
    """Every case returns on the host checks; no pointer is dereferenced and nothing is launched."""
    lo = good()
    fb, mb, _ = kvc.chunk_sizes(lo)
    C = 1024
    dense = (2 * 4096 * C, 4096 * C, C)
    A = 0x7F0000000000  # an aligned, never dereferenced address

    def status(fn, *a):
        try:
            fn(*a)
        except kvc.KvcError as e:
            return e.status
        return 0

    assert status(kvc.kvc_pack, lo, None, dense, 4096, A, 2 * fb, A, 2 * mb) == 1          # null input
    assert status(kvc.kvc_pack, lo, A, dense, 4096, A, 2 * fb - 1, A, 2 * mb) == 3         # frames too small
    assert status(kvc.kvc_pack, lo, A, dense, 4096, A, 2 * fb, A, mb) == 3                 # meta too small
    assert status(kvc.kvc_pack, lo, A, dense, -1, A, 2 * fb, A, 2 * mb) == 1               # negative count
    assert status(kvc.kvc_pack, lo, A + 2, dense, 4096, A, 2 * fb, A, 2 * mb) == 1         # misaligned input
    assert status(kvc.kvc_pack, lo, A, (dense[0], dense[1], C + 4), 4096, A, 2 * fb, A, 2 * mb) == 1  # stride % 8
    assert status(kvc.kvc_pack, lo, A, (dense[0], dense[1], C - 8), 4096, A, 2 * fb, A, 2 * mb) == 1  # tokens overlap
    assert status(kvc.kvc_pack, good(head_dim=4, num_kv_heads=256), A, dense, 4096, A, 2 * fb, A, 2 * mb) == 2
    assert status(kvc.kvc_pack, good(tile_w=4, tile_h=256), A, dense, 4096, A, 2 * fb, A, 2 * mb) == 2
    assert status(kvc.kvc_restore, lo, A, None, 4096, A, dense) == 1
    assert status(kvc.kvc_restore, lo, A, A + 4, 4096, A, dense) == 1                      # meta not 8-aligned
    # paged: first_token must be a chunk boundary, the table must cover the range
    paged = lambda **k: status(kvc.kvc_restore_paged, lo, A, A, k.get("first", 0), k.get("n", 4096), k.get("cache", A),
                               k.get("nb", 256), k.get("bs", 16), k.get("table", A), k.get("tl", 256))
    assert paged(first=100) == 1
    assert paged(tl=255) == 1
    assert paged(first=2048, n=4096, tl=256) == 1
    assert paged(bs=0) == 1
    assert paged(nb=0) == 1
    assert paged(cache=None) == 1
    assert paged(table=None) == 1
    # pipeline
    chunks = [(A, kvc.blob_meta_offset(lo) + mb, 2048)] * 3
    blob = kvc.blob_meta_offset(lo) + mb
    pipe = lambda **k: status(kvc.kvc_fetch_pipeline, lo, k.get("chunks", chunks), k.get("staging", [A, A + 256]),
                              k.get("sb", blob), A, 512, 16, A, k.get("tl", 512), None, k.get("cs", 1), k.get("xs", 2))
    assert pipe(staging=[A]) == 1                          # one staging slot: neither staged nor in place
    assert pipe(staging=[], chunks=[(A + 4, blob, 2048)]) == 1   # in place: the kernel loads 8 bytes at a time
    assert pipe(staging=[], xs=0) == 1
    assert pipe(staging=[], chunks=[(A, blob - 1, 2048)]) == 3
    assert pipe(sb=blob - 1) == 3
    assert pipe(chunks=[(A, blob - 1, 2048)]) == 3
    assert pipe(chunks=[(A, blob, 100), (A, blob, 2048)]) == 1   # only the last chunk may be short
    assert pipe(chunks=[(A, blob, 0)]) == 1
    assert pipe(cs=5, xs=5) == 1                           # one stream for both roles
    assert pipe(cs=0) == 1
    assert pipe(tl=10) == 1
    assert pipe(staging=[A, A + 8]) == 1                   # staging alignment


def test_frame_calls_reject_bad_arguments(kvc_lib):
    lo = good()
    fb, mb, F = kvc.chunk_sizes(lo)
    A = 0x7F0000000000
    assert kvc.frame_size(lo) == 3 * 512 * 1024
    assert kvc.frame_offset(lo, 0, 0, 0) == 0 and kvc.frame_offset(lo, 1, 10, 3) == fb - kvc.frame_size(lo)
    bad = ctypes.c_size_t(-1).value
    assert kvc.frame_offset(lo, 2, 0, 0) == bad and kvc.frame_offset(lo, 0, 11, 0) == bad and kvc.frame_offset(lo, 0, 0, 4) == bad

    def status(fn, *a):
        try:
            fn(*a)
        except kvc.KvcError as e:
            return e.status
        return 0

    fr = lambda **k: status(kvc.kvc_restore_paged_frame, lo, k.get("frame", A), k.get("meta", A), k.get("kind", 0),
                            k.get("lg", 0), k.get("f", 0), k.get("first", 0), k.get("n", 2048), A, 256, 16, A,
                            k.get("tl", 256))
    assert fr(kind=2) == 1 and fr(lg=11) == 1 and fr(f=4) == 1 and fr(f=-1) == 1
    assert fr(first=7) == 1 and fr(n=0) == 1 and fr(n=2049) == 1 and fr(tl=100) == 1
    assert fr(frame=None) == 1 and fr(meta=None) == 1 and fr(frame=A + 4) == 1
    frs = lambda first, count: status(kvc.kvc_restore_paged_frames, lo, A, A, first, count, 0, 2048, A, 256, 16, A, 256)
    assert frs(-1, 1) == 1 and frs(0, 0) == 1 and frs(88, 1) == 1 and frs(80, 9) == 1 and frs(0, 89) == 1
    blob = kvc.blob_meta_offset(lo) + mb
    chunks = [(A, blob, 2048)] * 2
    fsz = kvc.frame_size(lo)
    pipe = lambda **k: status(kvc.kvc_fetch_pipeline_frames, lo, k.get("chunks", chunks), k.get("fst", [A, A + 256]),
                              k.get("fsb", fsz), k.get("mst", [A, A + 256]), k.get("msb", mb), A, 512, 16, A, 512, None,
                              k.get("cs", 1), k.get("xs", 2), k.get("order", 0), k.get("ev", None))
    assert pipe(fst=[A]) == 1 and pipe(mst=[A]) == 1
    assert pipe(fsb=fsz - 1) == 3 and pipe(msb=mb - 1) == 3
    assert pipe(chunks=[(A, blob - 1, 2048)]) == 3
    assert pipe(cs=3, xs=3) == 1 and pipe(fst=[A, A + 8]) == 1
    assert pipe(order=2) == 1 and pipe(order=-1) == 1
    assert pipe(ev=[A] * 10 + [None]) == 1
    # in place (no frame staging): misaligned blob, missing compute stream, short blob
    assert pipe(fst=[], mst=[], chunks=[(A + 4, blob, 2048)]) == 1
    assert pipe(fst=[], mst=[], xs=0) == 1
    assert pipe(fst=[], mst=[], chunks=[(A, blob - 1, 2048)]) == 3
    # meta staging: a chunk section, or the pairs of three layers (K per channel, V per token and head)
    assert kvc.meta_staging_size(lo, kvc.KVC_ORDER_CHUNK) == mb
    slice_bytes = 3 * (8 * 128 + 2048 * 8) * 8
    assert kvc.meta_staging_size(lo, kvc.KVC_ORDER_LAYER) == slice_bytes
    assert kvc.meta_staging_size(lo, 2) == bad
    assert pipe(order=1, msb=slice_bytes - 1) == 3


def test_admission_matches_oracle(kvc_lib):
    """Appx A.3 condition: the library's running-sum form against the oracle's one-inequality-per-stage form."""
    from oracle import admission
    rng = np.random.default_rng(11)
    for case in range(300):
        n = int(rng.integers(1, 40))
        if case % 3 == 0:      # integer times: ties (equality) are hit often
            f, c = rng.integers(0, 4, n).tolist(), rng.integers(0, 5, n).tolist()
        else:
            f, c = rng.uniform(0, 1, n).tolist(), rng.uniform(0, 1.6, n).tolist()
        assert kvc.admission_min_buffered(f, c) == admission.min_buffered(f, c)
        for b in range(n + 1):
            assert kvc.admission_ok(f, c, b) == int(admission.condition_holds(f, c, b))
    assert kvc.admission_ok([1.0], [1.0], 2) == -1 and kvc.admission_ok([1.0], [1.0], -1) == -1
    assert kvc.admission_ok([-1.0], [1.0], 0) == -1 and kvc.admission_ok([1.0], [float("nan")], 0) == -1
    assert kvc.admission_min_buffered([float("inf")], [1.0]) == -1 and kvc.admission_min_buffered([], []) == -1
    assert kvc.load().kvc_admission_ok(None, None, 1, 0) == -1


def test_status_strings(kvc_lib):
    assert kvc.status_str(0) == "ok"
    assert {kvc.status_str(i) for i in range(5)}.isdisjoint({"unknown status"})
    assert kvc.status_str(99) == "unknown status"


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load(str(tmp_path / "libkvc.so"))


def test_select_resolution_matches_oracle_and_the_papers_tables(kvc_lib):
    """Alg. 1: the library against the oracle on random profile tables and on the hand-evaluated cases."""
    from oracle import resolution
    from test_oracle_pins import load_alg1_cases, load_alg1_tables
    tables = load_alg1_tables()
    for dev, load, active, bw, chosen, bubble in load_alg1_cases():
        sizes, rows, pen = tables[dev]
        r, b = kvc.select_resolution(sizes, rows, pen, load, active, bw)
        assert r == chosen and abs(b - bubble) < 1e-8
    rng = np.random.default_rng(21)
    for case in range(300):
        n, loads = int(rng.integers(1, 7)), int(rng.integers(1, 8))
        if case % 3 == 0:   # small integers: exact ties and zero bubbles
            sizes, lat, pen = rng.integers(1, 6, n) * 100.0, rng.integers(0, 6, (loads, n)) * 1.0, rng.integers(0, 2, n) * 1.0
            bw = 100.0
        else:
            sizes, lat, pen = rng.uniform(50, 300, n), rng.uniform(0.05, 0.6, (loads, n)), rng.uniform(0, 0.1, n)
            bw = float(rng.uniform(100, 2000))
        load, active = int(rng.integers(1, loads + 1)), int(rng.integers(-1, n))
        want = resolution.select_resolution(sizes, lat, pen, load, active, bw)
        assert kvc.select_resolution(sizes.tolist(), lat.tolist(), pen.tolist(), load, active, bw) == want
    s, l, p = [180.0, 256.0], [[0.2, 0.19]], [0.08, 0.0]
    assert kvc.select_resolution(s, l, p, 0, 0, 100.0)[0] == -1 and kvc.select_resolution(s, l, p, 2, 0, 100.0)[0] == -1
    assert kvc.select_resolution(s, l, p, 1, 2, 100.0)[0] == -1 and kvc.select_resolution(s, l, p, 1, -2, 100.0)[0] == -1
    assert kvc.select_resolution(s, l, p, 1, 0, 0.0)[0] == -1 and kvc.select_resolution(s, l, p, 1, 0, float("nan"))[0] == -1
    assert kvc.select_resolution([180.0, -1.0], l, p, 1, 0, 100.0)[0] == -1
    assert kvc.select_resolution(s, [[0.2, float("inf")]], p, 1, 0, 100.0)[0] == -1
    assert kvc.est_bandwidth(256e6, 0.5) == resolution.est_bandwidth(256e6, 0.5) == 512e6
    assert kvc.est_bandwidth(1.0, 0.0) == -1.0 and kvc.est_bandwidth(-1.0, 1.0) == -1.0


def test_layout_set_resolution(kvc_lib):
    """The paper's four resolutions as tile grids of the (8,128) tile: whole tiles inside width x height."""
    for (wd, ht), (tx, ty, F) in {(426, 240): (3, 30, 23), (854, 480): (6, 60, 6), (1138, 640): (8, 80, 4),
                                  (1920, 1080): (15, 135, 2)}.items():
        lo = good()
        assert kvc.layout_set_resolution(lo, wd, ht) == 0
        assert (lo.tiles_x, lo.tiles_y) == (tx, ty)
        fb, mb, frames = kvc.chunk_sizes(lo)
        assert frames == F and fb == 2 * 11 * F * 3 * (ty * 8) * (tx * 128)
    lo = good()
    assert kvc.layout_set_resolution(lo, 100, 4) == 0 and (lo.tiles_x, lo.tiles_y) == (1, 1)   # smaller than a tile
    assert kvc.layout_set_resolution(lo, 0, 240) == 1 and kvc.layout_set_resolution(lo, 426, -1) == 1


def test_bench_contract_pieces_that_need_no_gpu():
    """bench.py: algorithmic bytes of the benchmark workload (1 code byte + 2 output bytes + pairs per element for
    restore; 2 input bytes + every frame byte + pairs for pack) and the refusal of more than one GPU."""
    import subprocess
    import sys

    import bench
    import kv_synth
    w = kv_synth.WORKLOADS["llama3_8b_32k_paged"]
    fb, mb, _ = kvc.chunk_sizes(good())
    elems, pack_bytes, restore_bytes = bench.algorithmic_bytes(w, fb, mb)
    assert elems == 32 * 2 * 32768 * 1024
    pairs = 16 * (32 * 1024 + 32 * 2048 * 8) * 8              # per chunk: K per channel, V per (token, head)
    assert restore_bytes == 3 * elems + pairs == 6_513_754_112
    assert pack_bytes == 2 * elems + 16 * fb + pairs == 6_580_862_976
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one GPU" in r.stderr and r.stdout == ""


def test_pack_keeps_strips_resident_only_while_32_bit_row_offsets_hold(kvc_lib):
    """The register-resident body of kvc_pack addresses all 2048 token rows of a strip with 32-bit byte offsets,
    whatever the chunk length: a short chunk with a huge token stride (token-major engine tensors) must take the
    streaming body instead."""
    C = 1024
    dense = (2 * 4096 * C, 4096 * C, C)
    assert kvc.pack_plan(good(), dense) == (1, 512)
    assert kvc.pack_plan(good(chunk_tokens=1024, tiles_y=32), dense)[0] == 1
    assert kvc.pack_plan(good(chunk_tokens=4096, tiles_y=128), dense)[0] == 0          # chunk longer than a strip
    assert kvc.pack_plan(good(k_mode=1), dense)[0] == 0                                 # nothing per channel
    # token-major [token][L][2][H][D] with 80 layers of 8192 channels: 2.6 MB between tokens
    big = good(num_layers=80, num_kv_heads=64, tile_h=64, chunk_tokens=1024, tiles_y=32)
    Cb = 64 * 128
    ts = 80 * 2 * Cb
    assert 1023 * ts * 2 < 2**32 < 2047 * ts * 2   # the chunk's own rows fit, the strip's 2048 rows do not
    assert kvc.pack_plan(big, (2 * Cb, Cb, ts))[0] == 0
    # just below / at the limit: 2048 rows * ts * 2 bytes < 2^32
    edge = 2**32 // (2048 * 2)
    assert kvc.pack_plan(good(), (8, 8, edge - 8))[0] == 1
    assert kvc.pack_plan(good(), (8, 8, edge))[0] == 0
    with pytest.raises(kvc.KvcError):
        kvc.pack_plan(good(), (0, 0, C - 8))


def test_tile_candidates_equal_the_oracles_enumeration(kvc_lib):
    from oracle import residuals as R

    for H, D in [(8, 128), (32, 128), (1, 8), (6, 16), (40, 96)]:
        assert kvc.tile_candidates(H, D) == R.tile_candidates(H, D)
    for th, tw, seg in kvc.tile_candidates(8, 128):
        assert kvc.layout_validate(good(tile_h=th, tile_w=tw, tile_seg=seg)) == 0
    assert kvc_lib.kvc_tile_candidates(0, 128, None, None, None, 0) == -1
    assert kvc_lib.kvc_tile_candidates(8, 128, None, None, None, 4) == -1


def test_proxy_cost_equals_the_oracle_on_random_histograms(kvc_lib, oracle):
    """kvc_proxy_cost_bits is host arithmetic: same histograms in, same bits out as oracle/residuals.py (both sum
    -n log2(n/N) in double; the summation order differs, hence a relative tolerance of 1e-12)."""
    from oracle import residuals as R

    rng = np.random.default_rng(5)
    for kw, n_chunks in ((dict(num_layers=3, chunk_tokens=40, tiles_x=2, tiles_y=5), 2),
                         (dict(num_layers=2, chunk_tokens=16, tiles_x=4, tiles_y=4), 1)):    # F = 4 and F = 1
        lo = good(**kw)
        olo = oracle.make_layout(lo.num_layers, 8, 128, 0, lo.chunk_tokens, 8, 128, lo.tiles_x, lo.tiles_y)
        shape = (n_chunks, 2, lo.num_layers, R.N_RESIDUALS, 256)
        hist = rng.integers(0, 1000, size=shape).astype(np.uint64)
        hist[0, 0, 0, 0] = 0
        hist[0, 0, 0, 0, 17] = 12345            # a constant residual: entropy 0
        hist[0, 1, 1, 2] = 0                    # an empty histogram
        assert kvc.residual_histograms_size(lo, n_chunks) == hist.nbytes
        got = kvc.proxy_cost_bits(lo, hist.ctypes.data, n_chunks)
        want = R.total_cost_bits(olo, hist)
        assert abs(got - want) <= 1e-12 * want
    assert kvc.proxy_cost_bits(good(), None, 1) < 0


def test_residual_histograms_reject_bad_arguments(kvc_lib):
    lo = good()
    A = 0x7F0000000000
    need = kvc.residual_histograms_size(lo, 2)
    assert need == 2 * 2 * 32 * 5 * 256 * 8
    for args, status in (((A, 2, A, need - 8), 3), ((0, 2, A, need), 1), ((A, 2, 0, need), 1), ((A + 4, 2, A, need), 1),
                         ((A, -1, A, need), 1)):
        with pytest.raises(kvc.KvcError) as e:
            kvc.kvc_residual_histograms(lo, *args)
        assert e.value.status == status
    kvc.kvc_residual_histograms(lo, A, 0, A, 0)   # nothing to do: returns before anything is enqueued


def test_probe_expand_rejects_bad_arguments(kvc_lib):
    A = 0x7F0000000000
    ok = dict(out=1 << 20, mp=0, piece=32768, wg=4096, shape=0)
    for kw, status in ((dict(wg=8192), 1), (dict(piece=4096), 1), (dict(piece=48 * 1024), 1), (dict(out=(1 << 20) + 4096), 1),
                       (dict(src=0), 1), (dict(dst=A + 8), 1), (dict(mp=A + 2), 1), (dict(shape=4), 1),
                       (dict(shape=1, wg=32768), 1), (dict(shape=2, wg=32768), 1)):
        a = dict(ok, src=A, dst=A)
        a.update(kw)
        with pytest.raises(kvc.KvcError) as e:
            kvc.kvc_probe_expand(a["src"], a["dst"], a["out"], a["mp"], a["piece"], a["wg"], shape=a["shape"])
        assert e.value.status == status, kw
    kvc.kvc_probe_expand(A, A, 0, 0, 32768, 4096)   # nothing to do
