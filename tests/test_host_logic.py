"""CPU-only tests of the HIP library's host side: it loads, exports what
include/sfc.h declares, validates arguments without touching a GPU, and its add
networks (compiled for the host) realize the oracle's matrices."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

from oracle import sfc as oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "sfc.h")


@pytest.fixture(scope="module")
def lib():
    from paper_2407_02913_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__ as entry

        entry.build()
    return binding.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sfc_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_three_named_entry_points():
    names = declared_functions()
    for must in ("sfc_plan", "sfc_transform_filter", "sfc_conv2d_nchw"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    from paper_2407_02913_amd import binding

    names = declared_functions()
    assert sorted(binding.EXPORTS) == names
    for n in names:
        assert hasattr(lib, n), n


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2407_02913_amd import binding

    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "nope.so"))
    monkeypatch.setattr(binding, "_lib", None)
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load()


def make_desc(**kw):
    from paper_2407_02913_amd import binding

    base = dict(N=2, Cin=16, Cout=24, H=14, W=9, alg=0, mode=1, out=0, path=0, per_channel_wscale=1,
                transform_bits=0, flags=0)
    base.update(kw)
    return binding.ConvDesc(**base)


def plan_status(lib, desc):
    h = C.c_void_p()
    st = lib.sfc_plan(C.byref(desc), C.byref(h))
    return st, h


def test_plan_sizes_and_counts(lib):
    st, h = plan_status(lib, make_desc())
    assert st == 0
    fb, wb, p, t = C.c_size_t(), C.c_size_t(), C.c_int32(), C.c_int64()
    assert lib.sfc_plan_sizes(h, C.byref(fb), C.byref(wb), C.byref(p), C.byref(t)) == 0
    th, tw = oracle.tile_grid(14, 9)
    assert p.value == oracle.multiplications_per_tile("6x6_p88") == 88
    assert t.value == 2 * th * tw
    tp, cp, kp = -(-t.value // 16) * 16, 64, 32
    assert fb.value >= 88 * kp * cp + 2 * 88 * kp * 4
    assert wb.value >= 88 * tp * cp + 88 * tp * kp * 4
    assert lib.sfc_plan_sizes(h, None, None, None, None) == 0
    lib.sfc_plan_destroy(h)
    st, h = plan_status(lib, make_desc(alg=1, mode=0))
    assert st == 0
    assert lib.sfc_plan_sizes(h, C.byref(fb), C.byref(wb), C.byref(p), C.byref(t)) == 0
    assert p.value == 100 and fb.value >= 100 * kp * cp * 2
    lib.sfc_plan_destroy(h)


@pytest.mark.parametrize(
    "kw,code",
    [
        (dict(N=0), 1), (dict(Cin=-1), 1), (dict(H=0), 1), (dict(alg=10), 1), (dict(alg=-2), 1),
        (dict(mode=2), 1), (dict(out=5), 1), (dict(path=3), 1), (dict(path=-2), 1),
        (dict(per_channel_wscale=2), 1), (dict(flags=2), 1),
        (dict(transform_bits=1), 1), (dict(transform_bits=9), 1),
        (dict(transform_bits=4, mode=0), 2),  # exact mode has no transform-domain rounding
        (dict(out=1, mode=1), 2),  # raw integer output only in exact mode
        (dict(path=1, mode=0), 2),  # fused path is the requantized one
        (dict(W=5000), 2),
        # exact mode keeps 32-bit sums: guaranteed up to 404 channels (3x3), 145 (5x5 filters),
        # 74 (7x7 filters)
        (dict(mode=0, Cin=405), 2), (dict(mode=0, alg=6, Cin=146), 2), (dict(mode=0, alg=8, Cin=75), 2),
        (dict(Cout=65521), 2),  # one workgroup row per (padded) filter must fit a launch grid
    ],
)
def test_plan_rejects_bad_descriptions(lib, kw, code):
    st, h = plan_status(lib, make_desc(**kw))
    assert st == code and not h.value


def test_exact_mode_channel_bound_and_its_opt_in(lib):
    for kw in (dict(mode=0, Cin=404), dict(mode=0, alg=6, Cin=145), dict(mode=0, alg=9, Cin=74),
               dict(mode=0, Cin=512, flags=1),
               dict(mode=1, Cin=512)):
        st, h = plan_status(lib, make_desc(**kw))
        assert st == 0, kw
        lib.sfc_plan_destroy(h)


def test_auto_algorithm_and_path(lib):
    """SFC_ALG_AUTO / SFC_PATH_AUTO: the library's choice per layer shape, reported by
    sfc_plan_choice; an explicit choice is kept.  The ResNet shapes and the 13-layer stack get
    what bench.py runs (it asks for auto and reads the choice back)."""
    from paper_2407_02913_amd import binding, synth

    def choice(shape, **kw):
        plan = binding.Plan(shape.N, shape.Cin, shape.Cout, shape.H, shape.W, **kw)
        got = (plan.alg, plan.path)
        plan.close()
        return got

    want = {"tiny32": ("4x4_p46", "single"), "resnet56": ("4x4_p46", "single"),
            "resnet28": ("4x4_p46", "single"), "resnet14": ("4x4_p46", "fused"),
            "resnet7": ("7x7_p132", "staged"), "cifar16": ("4x4_p46", "single"),
            "cifar8": ("4x4_p46", "fused")}
    for name, shape in synth.LAYERS.items():
        assert choice(shape, alg="auto", path="auto") == want[name], name
    assert choice(synth.LAYERS["resnet56"], alg="6x6_p88", path="staged") == ("6x6_p88", "staged")
    assert choice(synth.LAYERS["resnet56"], alg="7x7_p132", path="auto") == ("7x7_p132", "single")
    # 512 channels on 7x7 maps: one 7x7 tile per image through the batched GEMMs from batch 128 on
    r7 = synth.LAYERS["resnet7"]
    assert choice(synth.LayerShape("b128", 128, r7.Cin, r7.Cout, 7, 7, "relu", True, 9), alg="auto",
                  path="auto") == ("7x7_p132", "staged")
    assert choice(synth.LayerShape("b64", 64, r7.Cin, r7.Cout, 7, 7, "relu", True, 9), alg="auto",
                  path="auto") == ("4x4_p46", "fused")
    # exact mode runs staged, on the 6x6 form the paper's headline count is about
    assert choice(synth.LAYERS["tiny32"], alg="auto", path="auto", mode="exact") == ("6x6_p88", "staged")
    # channel counts the fused kernel does not take (three 64-channel slices) fall back
    odd = synth.LayerShape("odd", 2, 192, 32, 14, 14, "relu", True, 9)
    assert choice(odd, alg="auto", path="auto")[1] == "staged"
    for shape in synth.stack_layers():
        alg, path = choice(shape, alg="auto", path="auto", out="i8")
        assert alg == binding.AUTO_ALG_3X3
        assert path == ("single" if shape.Cin <= binding.SINGLE_MAX_CIN else "fused")


def test_undersized_buffers_are_refused_before_any_launch(lib):
    """Every call that takes a caller-owned device buffer takes its size and returns
    SFC_EWORKSPACE when it is too small (no GPU here: a launch would fail differently)."""
    st, h = plan_status(lib, make_desc())
    assert st == 0
    fb, wb = C.c_size_t(), C.c_size_t()
    assert lib.sfc_plan_sizes(h, C.byref(fb), C.byref(wb), None, None) == 0
    p = 88
    sx = (C.c_float * p)(*([0.5] * p))
    sw = (C.c_float * (p * 24))(*([0.25] * (p * 24)))
    assert lib.sfc_set_point_scales(h, sx, sw) == 0
    ws = (C.c_float * 24)(*([0.01] * 24))
    dev = C.c_void_p(4096)
    assert lib.sfc_transform_filter(h, dev, ws, dev, fb.value - 1, None) == 6
    assert lib.sfc_conv2d_nchw(h, dev, C.c_float(1.0), dev, dev, wb.value - 1, None) == 6
    assert lib.sfc_conv2d_stages(h, dev, C.c_float(1.0), dev, dev, 0, None, 7) == 6
    out = (C.c_float * (p * 24))()
    assert lib.sfc_calibrate_act_scales(h, dev, 1, dev, wb.value - 1, None, out) == 6
    assert lib.sfc_calibrate_filter_scales(h, dev, dev, wb.value - 1, None, out) == 6
    # large enough: the next check in line answers (the filter has not been transformed)
    assert lib.sfc_conv2d_nchw(h, dev, C.c_float(1.0), dev, dev, wb.value, None) == 4
    assert lib.sfc_status_string(6) == b"device buffer smaller than the plan needs"
    lib.sfc_plan_destroy(h)


def test_null_and_order_errors_without_gpu(lib):
    assert lib.sfc_plan(None, None) == 1
    st, h = plan_status(lib, make_desc())
    assert st == 0
    p = 88
    sx = (C.c_float * p)(*([0.5] * p))
    sw = (C.c_float * (p * 24))(*([0.25] * (p * 24)))
    assert lib.sfc_set_point_scales(h, None, sw) == 1
    bad = (C.c_float * p)(*([0.5] * (p - 1) + [0.0]))
    assert lib.sfc_set_point_scales(h, bad, sw) == 1
    nan = (C.c_float * p)(*([0.5] * (p - 1) + [float("nan")]))
    assert lib.sfc_set_point_scales(h, nan, sw) == 1
    assert lib.sfc_set_point_scales(h, sx, sw) == 0
    # conv before the filter transform, and misaligned / null pointers: rejected before any launch
    big = C.c_size_t(1 << 40)
    assert lib.sfc_conv2d_nchw(h, C.c_void_p(256), C.c_float(1.0), C.c_void_p(512), C.c_void_p(1024), big, None) == 4
    assert lib.sfc_conv2d_nchw(h, None, C.c_float(1.0), C.c_void_p(512), C.c_void_p(1024), big, None) == 1
    assert lib.sfc_conv2d_nchw(h, C.c_void_p(257), C.c_float(1.0), C.c_void_p(512), C.c_void_p(1024), big, None) == 1
    assert lib.sfc_conv2d_nchw(h, C.c_void_p(256), C.c_float(-1.0), C.c_void_p(512), C.c_void_p(1024), big, None) == 1
    ws = (C.c_float * 24)(*([0.01] * 24))
    assert lib.sfc_transform_filter(h, C.c_void_p(3), ws, C.c_void_p(512), big, None) == 1
    lib.sfc_plan_destroy(h)
    # requantized mode needs its scales before the filter transform
    st, h = plan_status(lib, make_desc())
    assert lib.sfc_transform_filter(h, C.c_void_p(256), ws, C.c_void_p(512), big, None) == 4
    lib.sfc_plan_destroy(h)
    # exact-mode plans take no point scales
    st, h = plan_status(lib, make_desc(mode=0))
    assert lib.sfc_set_point_scales(h, sx, sw) == 2
    lib.sfc_plan_destroy(h)
    assert lib.sfc_status_string(0) == b"ok" and lib.sfc_status_string(4) == b"scales or filter not set"


@pytest.fixture(scope="module")
def kernel_maps(tmp_path_factory):
    """The linear maps realized by the kernels' add networks, compiled for the host."""
    exe = tmp_path_factory.mktemp("host") / "points_check"
    src = os.path.join(ROOT, "tests", "host", "points_check.cpp")
    subprocess.run(["/opt/rocm/bin/hipcc", "--cuda-host-only", "-O1", "-std=c++17", src, "-o", str(exe)],
                   check=True, capture_output=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    maps = {}
    for line in out.splitlines():
        kind, alg, p, *vals = line.split()
        maps.setdefault((kind, int(alg)), {})[int(p)] = [int(v) for v in vals]
    return {k: np.array([v[i] for i in range(len(v))]) for k, v in maps.items()}


@pytest.mark.parametrize("alg_id,alg", [(0, "6x6_p88"), (1, "6x6_p100"), (2, "7x7_p132"), (3, "7x7_p144"),
                                        (4, "4x4_p46"), (5, "4x4_p49"),
                                        (6, "6x6_5x5_p184"), (7, "6x6_5x5_p196"),
                                        (8, "4x4_7x7_p184"), (9, "4x4_7x7_p196")])
def test_kernel_add_networks_realize_the_oracle_matrices(kernel_maps, alg_id, alg):
    b2, g2, a2, den = oracle.algorithm(alg)
    assert den == (16 if alg in ("4x4_p46", "4x4_p49") else 36)
    assert np.array_equal(kernel_maps[("B", alg_id)], b2)
    assert np.array_equal(kernel_maps[("G", alg_id)], g2)
    assert np.array_equal(kernel_maps[("A", alg_id)], a2)
    # the streaming form of the fused kernels (processing order + per-group collapse)
    assert np.array_equal(kernel_maps[("S", alg_id)], a2)


def test_bench_operation_counts_match_the_add_networks(tmp_path):
    """bench.py's vector-ALU roofline counts: recounted from sfc_points.hpp with a counting type."""
    import bench

    exe = tmp_path / "op_count"
    src = os.path.join(ROOT, "tests", "host", "op_count.cpp")
    subprocess.run(["/opt/rocm/bin/hipcc", "--cuda-host-only", "-O1", "-std=c++17", src, "-o", str(exe)],
                   check=True, capture_output=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    names = ["6x6_p88", "6x6_p100", "7x7_p132", "7x7_p144", "4x4_p46", "4x4_p49"]
    for line in out.splitlines():
        alg, pts, in_adds, out_ops = (int(v) for v in line.split())
        assert pts == oracle.multiplications_per_tile(names[alg])
        assert bench.ADD_NETWORK_OPS[names[alg]] == (in_adds, out_ops)
    # the 6x6 input network is the paper's: 14 additions per symbolic DFT-6 plus the correction
    # inputs, 16 per 1-D pass over 8 + 8 lines, plus the sums of the product rule
    assert bench.ADD_NETWORK_OPS["6x6_p88"][0] == 16 * 16 + 48


def test_group_scales_matches_the_oracle_for_every_granularity(lib):
    """Host-only entry point: the ablation's scale groupings against the oracle's."""
    from paper_2407_02913_amd import binding

    rng = np.random.default_rng(5)
    plan = binding.Plan(2, 16, 24, 14, 9, alg="6x6_p88", mode="requant")
    sx = rng.uniform(0.1, 4.0, size=plan.P).astype(np.float32)
    sw = rng.uniform(0.1, 4.0, size=(plan.P, 24)).astype(np.float32)
    for act in ("tensor", "point"):
        for filt in ("channel", "point", "channel_point"):
            gx, gw = plan.group_scales(sx, sw, act, filt)
            ox, ow = oracle.group_scales(sx, sw, act, filt)
            assert np.array_equal(gx, ox) and np.array_equal(gw, ow), (act, filt)
    h = plan._h
    fx, fw = (C.c_float * plan.P)(), (C.c_float * (plan.P * 24))()
    assert lib.sfc_group_scales(h, 2, 0, fx, fw) == 1 and lib.sfc_group_scales(h, 0, 3, fx, fw) == 1
    assert lib.sfc_group_scales(h, 0, 0, None, fw) == 1
    plan.close()
