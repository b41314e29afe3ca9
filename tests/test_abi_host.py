"""Host-side checks of the C ABI that need no GPU: the library loads, exports every
symbol include/camera.h declares, and rejects bad arguments before any GPU call."""
import ctypes
import os
import re

import pytest

from paper_2508_02322_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
vp, i64 = ctypes.c_void_p, ctypes.c_int64


@pytest.fixture(scope="module")
def lib():
    return binding.load_library()


@pytest.fixture()
def ctx(lib):
    c = vp()
    assert lib.camera_create(ctypes.byref(c), 0) == 0   # touches no GPU
    yield c
    lib.camera_destroy(c)


def declared_functions():
    text = open(os.path.join(ROOT, "include", "camera.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(camera_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert set(names) == set(binding.EXPORTS)
    for name in names:
        assert hasattr(lib, name), name
    assert lib.camera_version() == 1


def err(lib, ctx):
    return lib.camera_last_error(ctx).decode()


FAKE = vp(0x1000)   # aligned, never dereferenced: every call below fails validation first


def route(lib, ctx, **kw):
    a = dict(X=FAKE, dtype=1, n=16, d=64, ldx=64, W=FAKE, ldr=64, bias=None, ne=8, k=2, renorm=1, idx=FAKE, w=FAKE)
    a.update(kw)
    return lib.camera_route_topk(ctx, None, a["X"], a["dtype"], a["n"], a["d"], a["ldx"], a["W"], a["ldr"], a["bias"],
                                 a["ne"], a["k"], a["renorm"], a["idx"], a["w"])


def test_route_argument_checks(lib, ctx):
    assert lib.camera_route_topk(None, None, FAKE, 1, 16, 64, 64, FAKE, 64, None, 8, 2, 1, FAKE, FAKE) == -1
    assert route(lib, ctx, dtype=7) == -3 and "dtype" in err(lib, ctx)
    assert route(lib, ctx, n=-1) == -1 and "n:" in err(lib, ctx)
    assert route(lib, ctx, d=60) == -2 and "d_model" in err(lib, ctx)
    assert route(lib, ctx, ldx=32) == -2 and "ldx" in err(lib, ctx)
    assert route(lib, ctx, X=None) == -1 and "X" in err(lib, ctx)
    assert route(lib, ctx, X=vp(0x1004)) == -2 and "aligned" in err(lib, ctx)
    assert route(lib, ctx, ne=0) == -6 and "n_experts" in err(lib, ctx)
    assert route(lib, ctx, ne=257) == -6
    assert route(lib, ctx, k=9) == -1 and "top_k" in err(lib, ctx)
    assert route(lib, ctx, k=0) == -1
    assert route(lib, ctx, W=None) == -1 and "W_r" in err(lib, ctx)
    assert route(lib, ctx, idx=None) == -1 and "topk" in err(lib, ctx)
    assert route(lib, ctx, n=0) == 0          # empty input: nothing to do, no GPU needed


def score(lib, ctx, **kw):
    a = dict(X=FAKE, dtype=1, n=16, d=64, ldx=64, idx=FAKE, w=FAKE, k=2, ne=8, f=32, Wg=FAKE, Wu=FAKE, sgu=32 * 64,
             Wd=FAKE, sd=32 * 64, alpha=0.5, flags=0, p2=FAKE, pi=FAKE, o2=FAKE, en=FAKE)
    a.update(kw)
    return lib.camera_score_layer(ctx, None, a["X"], a["dtype"], a["n"], a["d"], a["ldx"], a["idx"], a["w"], a["k"],
                                  a["ne"], a["f"], a["Wg"], a["Wu"], a["sgu"], a["Wd"], a["sd"], a["alpha"], a["flags"],
                                  a["p2"], a["pi"], a["o2"], a["en"])


def test_score_argument_checks(lib, ctx):
    assert score(lib, ctx, w=None) == -1 and "both or neither" in err(lib, ctx)
    assert score(lib, ctx, k=0) == -1 and "top_k" in err(lib, ctx)
    assert score(lib, ctx, f=0) == -1 and "d_ff" in err(lib, ctx)
    assert score(lib, ctx, alpha=1.5) == -1 and "alpha" in err(lib, ctx)
    assert score(lib, ctx, alpha=float("nan")) == -1
    assert score(lib, ctx, flags=8) == -1 and "flags" in err(lib, ctx)
    assert score(lib, ctx, Wg=None) == -1 and "W_gate" in err(lib, ctx)
    assert score(lib, ctx, Wd=None) == -1 and "W_down" in err(lib, ctx)
    assert score(lib, ctx, en=None) == -1 and "energy" in err(lib, ctx)
    assert score(lib, ctx, p2=None) == -1 and "phi2" in err(lib, ctx)
    assert score(lib, ctx, sgu=100) == -2 and "stride_gu" in err(lib, ctx)
    assert score(lib, ctx, sd=100) == -2 and "stride_down" in err(lib, ctx)
    assert score(lib, ctx, ne=300) == -6
    assert score(lib, ctx, dtype=0, d=62) == -2
    assert score(lib, ctx, n=2 ** 31, k=2) == -2 and "pairs" in err(lib, ctx)
    assert score(lib, ctx, n=2 ** 24, k=8, ne=8) == -6 and "chunks" in err(lib, ctx)


def seg_array(vals):
    return (i64 * len(vals))(*vals)


def test_select_and_alloc_argument_checks(lib, ctx):
    sel = lambda **kw: lib.camera_select_prune(  # noqa: E731
        ctx, None, kw.get("E", FAKE), kw.get("n", 100), kw.get("seg", seg_array([0, 40, 100])), kw.get("n_seg", 2),
        kw.get("ratio", 0.4), kw.get("mask", FAKE), kw.get("per", FAKE), None, None)
    assert sel(E=None) == -1 and "energy" in err(lib, ctx)
    assert sel(n=-5) == -1
    assert sel(ratio=1.2) == -1 and "ratio" in err(lib, ctx)
    assert sel(ratio=-0.1) == -1
    assert sel(seg=seg_array([0, 40, 90])) == -1 and "seg_offsets" in err(lib, ctx)
    assert sel(seg=seg_array([0, 140, 100])) == -1 and "rising" in err(lib, ctx)
    assert sel(seg=seg_array([1, 40, 100])) == -1
    assert sel(n_seg=0) == -6 and "n_seg" in err(lib, ctx)
    assert sel(n_seg=513) == -6
    assert sel(seg=None) == -1
    assert sel(mask=None) == -1 and "keep_mask" in err(lib, ctx)
    assert sel(per=None) == -1 and "kept_per_expert" in err(lib, ctx)
    assert sel(E=vp(0x1008)) == -2

    def alloc(bits=(3, 2, 1), ratios=(0.1, 0.8, 0.1), n_levels=None, **kw):
        nl = len(bits) if n_levels is None else n_levels
        return lib.camera_alloc_bits(ctx, None, kw.get("E", FAKE), 100, seg_array([0, 40, 100]), 2, nl,
                                     (ctypes.c_int * len(bits))(*bits), (ctypes.c_double * len(ratios))(*ratios),
                                     kw.get("bit_of", FAKE), kw.get("lc", FAKE), None)
    assert alloc(ratios=(0.5, 0.2, 0.2)) == -1 and "sum to 1" in err(lib, ctx)
    assert alloc(ratios=(1.2, -0.1, -0.1)) == -1 and "negative" in err(lib, ctx)
    assert alloc(bits=(300, 2, 1)) == -1 and "bits" in err(lib, ctx)
    assert alloc(bits=(1,) * 9, ratios=(1.0,) + (0.0,) * 8) == -6 and "n_levels" in err(lib, ctx)
    assert alloc(n_levels=0) == -6
    assert alloc(lc=None) == -1 and "level_count" in err(lib, ctx)
    assert alloc(bit_of=None) == -1


def test_create_and_profile_checks(lib, ctx):
    assert lib.camera_create(None, 0) == -1
    c = vp()
    assert lib.camera_create(ctypes.byref(c), -3) == -1 and "device" in lib.camera_last_error(None).decode()
    assert lib.camera_destroy(None) == 0
    assert lib.camera_profile_enable(None, 1) == -1
    ms, cnt = ctypes.c_double(), i64()
    assert lib.camera_profile_read(ctx, 99, ctypes.byref(ms), ctypes.byref(cnt)) == -1
    assert lib.camera_profile_read(ctx, 0, None, ctypes.byref(cnt)) == -1


def test_bench_library_exports_and_argument_checks():
    """The machine probes live in a library of their own (include/camera_bench.h), not in the product ABI."""
    from paper_2508_02322_amd import bench_probes
    text = re.sub(r"/\*.*?\*/", "", open(os.path.join(ROOT, "include", "camera_bench.h")).read(), flags=re.S)
    assert sorted(set(re.findall(r"\b(camera_bench_[a-z0-9_]+)\s*\(", text))) == sorted(bench_probes.EXPORTS)
    blib = bench_probes.load_library()
    tf, mhz = ctypes.c_double(), ctypes.c_double()
    assert blib.camera_bench_mfma_bf16(0, 1, 0, ctypes.byref(tf), ctypes.byref(mhz)) == -1
    assert blib.camera_bench_mfma_bf16(0, 1, 1, None, ctypes.byref(mhz)) == -1
    assert blib.camera_bench_mfma_bf16(-1, 1, 1, ctypes.byref(tf), ctypes.byref(mhz)) == -1
    assert blib.camera_bench_hbm_read(0, 1000, 1, ctypes.byref(tf)) == -1
    assert blib.camera_bench_hbm_read(0, 1 << 30, 0, ctypes.byref(tf)) == -1
    assert blib.camera_bench_hbm_read(0, 1 << 30, 1, None) == -1
    assert not any(hasattr(binding.load_library(), n) for n in ("camera_probe_mfma_bf16", "camera_bench_mfma_bf16"))


def test_missing_library_fails_loudly(tmp_path):
    with pytest.raises(FileNotFoundError):
        binding.load_library(str(tmp_path / "libcamera_hip.so"))


def test_gather_argument_checks(lib, ctx):
    vpp = ctypes.c_void_p
    fake = vpp(4096)          # never dereferenced: every check below fails on the host
    def gather(dtype=1, n_experts=2, d_ff=64, d_model=16, wg=fake, wu=fake, stride_gu=64 * 16, wd=fake,
               stride_down=64 * 16, index=fake, n_index=10, base=0, count=fake, align=1, og=fake, ou=fake, od=fake, c=ctx):
        return lib.camera_gather_micro_experts(c, None, dtype, n_experts, d_ff, d_model, wg, wu, stride_gu, wd,
                                               stride_down, index, n_index, base, count, align, og, ou, od)
    assert gather(c=None) == -1
    assert gather(dtype=7) == -3
    assert gather(align=0) == -1 and gather(align=513) == -1 and "down_row_align" in err(lib, ctx)
    assert gather(n_experts=0) == -6 and gather(n_experts=257) == -6
    assert gather(d_ff=0) == -2
    assert gather(d_ff=40000, stride_gu=40000 * 16, stride_down=40000 * 16) == -6 and "65536" in err(lib, ctx)
    assert gather(d_model=12) == -2 and "16-byte" in err(lib, ctx)
    assert gather(n_index=-1) == -1 and gather(n_index=129) == -1
    assert gather(count=None, n_index=10) == -1 and "count" in err(lib, ctx)
    assert gather(wg=None) == -1 and "W_gate" in err(lib, ctx)
    assert gather(wd=None) == -1 and "W_down" in err(lib, ctx)
    assert gather(stride_gu=100) == -2 and gather(stride_down=100) == -2
    assert gather(og=vpp(4100)) == -2 and "aligned" in err(lib, ctx)
    assert gather(index=None) == -1 and "index" in err(lib, ctx)
    assert gather(base=-1) == -1
    assert gather(n_index=0) == 0                      # nothing to do
    assert gather(og=None, ou=None, od=None) == 0      # every output skipped


def test_layer_forward_and_output_error_argument_checks(lib, ctx):
    vpp = ctypes.c_void_p
    fake = vpp(4096)
    def forward(x=fake, dtype=1, n=16, d_model=64, ldx=64, idx=fake, w=fake, top_k=2, n_experts=4, d_ff=32, wg=fake,
                wu=fake, stride_gu=32 * 64, wd=fake, stride_down=32 * 64, keep=None, flags=0, y=fake, c=ctx):
        return lib.camera_layer_forward(c, None, x, dtype, n, d_model, ldx, idx, w, top_k, n_experts, d_ff, wg, wu,
                                        stride_gu, wd, stride_down, keep, flags, y)
    lib.camera_layer_forward.restype = ctypes.c_int
    assert forward(c=None) == -1
    assert forward(dtype=0, d_ff=30) == -2 and "multiple of 4" in err(lib, ctx)
    assert forward(dtype=9) == -3
    assert forward(idx=None) == -1 and "both or neither" in err(lib, ctx)
    assert forward(top_k=0) == -1 and forward(top_k=5) == -1
    assert forward(n_experts=0) == -6
    assert forward(d_ff=12) == -2 and "multiple of 8" in err(lib, ctx)
    assert forward(flags=2) == -1 and "flags" in err(lib, ctx)
    assert forward(wd=None) == -1
    assert forward(y=None) == -1 and "Y" in err(lib, ctx)
    assert forward(stride_gu=100) == -2 and forward(stride_down=100) == -2
    assert forward(y=vpp(4100)) == -2
    assert forward(n=0) == 0
    def error(y=fake, yh=fake, n=4, d=8, out=fake, c=ctx):
        return lib.camera_output_error(c, None, y, yh, n, d, out)
    assert error(c=None) == -1
    assert error(n=-1) == -2 and error(d=0) == -2
    assert error(y=None) == -1 and error(out=None) == -1
    assert error(n=0) == 0


def test_select_prune_multi_argument_checks(lib, ctx):
    fake = ctypes.c_void_p(4096)
    seg = (i64 * 3)(0, 50, 100)
    def multi(energy=fake, n=100, seg_=seg, n_seg=2, ratios=(0.2, 0.4), n_ratios=None, bits=fake, per=fake, c=ctx):
        arr = (ctypes.c_double * len(ratios))(*ratios) if ratios is not None else None
        return lib.camera_select_prune_multi(c, None, energy, n, seg_, n_seg, len(ratios) if n_ratios is None else n_ratios,
                                             arr, bits, per)
    assert multi(c=None) == -1
    assert multi(n_ratios=0) == -6 and multi(ratios=(0.1,) * 8) == -6
    assert multi(ratios=(0.4, 0.2)) == -1 and "fall" in err(lib, ctx)
    assert multi(ratios=(0.2, 1.5)) == -1
    assert multi(per=None) == -1 and multi(bits=None) == -1
    assert multi(n_seg=0) == -6


def test_layer_forward_compact_argument_checks(lib, ctx):
    fake = vp(4096)           # never dereferenced: every check below fails on the host

    def forward(x=fake, dtype=1, n=16, d_model=64, ldx=64, idx=fake, w=fake, top_k=2, n_experts=4, n_shared=0,
                count=(8, 9, 0, 31), align=1, wg=fake, wu=fake, wd=fake, flags=0, y=fake, c=ctx):
        counts = None if count is None else (ctypes.c_int32 * len(count))(*count)
        return lib.camera_layer_forward_compact(c, None, x, dtype, n, d_model, ldx, idx, w, top_k, n_experts, n_shared,
                                                counts, align, wg, wu, wd, flags, y)
    lib.camera_layer_forward_compact.restype = ctypes.c_int
    assert forward(c=None) == -1
    assert forward(dtype=0) == -6 and "BF16" in err(lib, ctx)
    assert forward(dtype=5) == -3
    assert forward(d_model=60) == -2
    assert forward(idx=None) == -1 and "both or neither" in err(lib, ctx)
    assert forward(idx=None, w=None, n_shared=1, count=(8, 9, 0, 31, 4)) == -1 and "n_shared" in err(lib, ctx)
    assert forward(n_shared=-1) == -1
    assert forward(n_experts=0, count=()) == -6
    assert forward(n_experts=250, n_shared=7, count=(1,) * 257) == -6 and "256" in err(lib, ctx)
    assert forward(top_k=0) == -1 and forward(top_k=5) == -1
    assert forward(flags=2) == -1 and "flags" in err(lib, ctx)
    assert forward(count=None) == -1 and "count" in err(lib, ctx)
    assert forward(count=(8, -1, 0, 31)) == -1 and "count[1]" in err(lib, ctx)
    assert forward(align=0) == -1 and forward(align=513) == -1 and "down_row_align" in err(lib, ctx)
    assert forward(wg=None) == -1 and "W_gate_c" in err(lib, ctx)
    assert forward(y=None) == -1 and "Y" in err(lib, ctx)
    assert forward(wd=vp(4100)) == -2 and "16-byte" in err(lib, ctx)
    assert forward(n=0) == 0                                  # nothing to do: no GPU is touched
    assert forward(count=(0, 0, 0, 0), wg=None, wu=None, wd=None, n=0) == 0


def test_select_prune_noalloc_argument_checks(lib, ctx):
    """The no-allocation variant refuses what does not fit its static scratch before any GPU call."""
    def sel(n=100, seg=None, n_seg=2, ratio=0.4, E=FAKE, mask=FAKE, per=FAKE, c=ctx):
        seg = seg_array([0, 40, n]) if seg is None else seg
        return lib.camera_select_prune_noalloc(c, None, E, n, seg, n_seg, ratio, mask, per, None)
    assert sel(c=None) == -1
    assert sel(n=(1 << 20) + 1) == -6 and "static scratch" in err(lib, ctx)
    assert sel(n=1 << 24) == -6
    assert sel(ratio=1.5) == -1 and "ratio" in err(lib, ctx)
    assert sel(E=None) == -1 and sel(mask=None) == -1 and sel(per=None) == -1
    assert sel(seg=seg_array([0, 40, 90])) == -1 and "seg_offsets" in err(lib, ctx)
    assert sel(n_seg=0) == -6


def test_rank_decisions_argument_checks(lib, ctx):
    seg = seg_array([0, 40, 100])

    def both(ratios=(0.2, 0.4), bits=(3, 2, 1), level_ratios=(0.2, 0.6, 0.2), n_ratios=None, n_levels=None, E=FAKE,
             keep=FAKE, per=FAKE, bit_of=FAKE, lc=FAKE, c=ctx):
        return lib.camera_rank_decisions(
            c, None, E, 100, seg, 2, len(ratios) if n_ratios is None else n_ratios,
            (ctypes.c_double * len(ratios))(*ratios), keep, per, len(bits) if n_levels is None else n_levels,
            (ctypes.c_int * len(bits))(*bits), (ctypes.c_double * len(level_ratios))(*level_ratios), bit_of, lc, None)
    assert both(c=None) == -1
    assert both(n_ratios=0) == -6 and both(n_levels=0) == -6
    assert both(ratios=(0.1,) * 6, bits=(3, 2, 1)) == -6 and "cuts" in err(lib, ctx)         # 6 + 2 cuts > 7
    assert both(ratios=(0.4, 0.2)) == -1 and "fall" in err(lib, ctx)
    assert both(level_ratios=(0.5, 0.2, 0.2)) == -1 and "sum to 1" in err(lib, ctx)
    assert both(bits=(300, 2, 1)) == -1
    assert both(per=None) == -1 and both(lc=None) == -1 and both(keep=None) == -1 and both(bit_of=None) == -1
    assert both(E=None) == -1 and "energy" in err(lib, ctx)


def test_input_channel_energy_argument_checks(lib, ctx):
    def energy(x=FAKE, dtype=1, n=16, d=64, ldx=64, idx=FAKE, k=2, ne=8, h=FAKE, c=ctx):
        return lib.camera_input_channel_energy(c, None, x, dtype, n, d, ldx, idx, k, ne, h)
    assert energy(c=None) == -1
    assert energy(dtype=9) == -3
    assert energy(d=60) == -2 and "d_model" in err(lib, ctx)
    assert energy(ne=0) == -6 and energy(ne=300) == -6
    assert energy(k=0) == -1 and energy(k=9) == -1 and "top_k" in err(lib, ctx)
    assert energy(h=None) == -1 and "h:" in err(lib, ctx)
    assert energy(x=None) == -1
