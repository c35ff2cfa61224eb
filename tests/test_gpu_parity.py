"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Integer stages (V, U, M taps, exact-mode sums) must be bit-exact; the dequantized
float32 output must be within 1e-5 of max|y_ref| of the oracle's float64 value."""
import numpy as np
import pytest

from oracle import sfc as oracle
from paper_2407_02913_amd import synth

pytestmark = pytest.mark.gpu

F32_TOL = 1e-5

SMALL_SHAPES = [  # (N, Cin, Cout, H, W)
    (1, 16, 16, 32, 32),  # the small workload: 36 tiles, ragged (32 = 5*6 + 2)
    (2, 3, 5, 14, 14),
    (1, 4, 4, 7, 7),
    (2, 2, 3, 13, 9),
    (1, 1, 1, 1, 1),  # degenerate: one pixel, one channel
    (1, 1, 2, 6, 6),  # exactly one full tile
    (3, 70, 40, 9, 20),  # Cin spans two 64-channel slices, Cout not a multiple of 16
    (5, 64, 64, 12, 18),  # 30 tiles: a ragged last 16-row block
]


@pytest.fixture(scope="module")
def binding():
    from paper_2407_02913_amd import binding as b

    b.load()
    return b


def uniform_case(shape, seed, r=3):
    n, c, k, h, w = shape
    rng = np.random.default_rng(seed)
    x = rng.integers(-128, 128, size=(n, c, h, w)).astype(np.int8)
    wt = rng.integers(-128, 128, size=(k, c, r, r)).astype(np.int8)
    ws = rng.uniform(0.005, 0.02, size=k).astype(np.float32)
    return x, wt, 0.02, ws


def rel_err(y, ref):
    return float(np.abs(y.astype(np.float64) - ref).max() / max(np.abs(ref).max(), 1e-30))


ALGS = ["6x6_p88", "6x6_p100", "7x7_p132", "7x7_p144"]
ALGS_STAGED = ALGS + ["4x4_p46", "4x4_p49"]  # SFC-4(4x4,3x3): staged and fused paths


@pytest.mark.parametrize("alg", ALGS_STAGED)
@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_exact_mode_taps_and_sums_bit_exact(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 100 + len(alg) + sum(shape))
    print("case exact", shape, alg, flush=True)
    acc_ref, taps_ref = oracle.conv_exact(x, w, alg, return_taps=True)
    assert np.array_equal(acc_ref, oracle.direct_conv(x, w))
    acc, taps = binding.conv2d(x, w, xs, ws, mode="exact", alg=alg, out="i32", return_taps=True)
    for name in ("V", "U", "M"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    assert np.array_equal(acc.astype(np.int64), acc_ref)
    y = binding.conv2d(x, w, xs, ws, mode="exact", alg=alg, out="f32")
    assert rel_err(y, oracle.dequantize(acc_ref, xs, ws)) <= F32_TOL


@pytest.mark.parametrize("alg", ALGS_STAGED)
@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_requant_mode_taps_bit_exact_and_output_close(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 200 + len(alg) + sum(shape))
    print("case requant", shape, alg, flush=True)
    # calibrate on different data so that some values clamp
    xc, _, _, _ = uniform_case(shape, 300 + sum(shape))
    sx = oracle.calibrate_act_scales(xc // 2, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, sx=sx, sw=sw, return_taps=True)
    for name in ("V", "U", "M"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    assert np.abs(taps["V"]).max() == 127  # the clamp was exercised
    assert rel_err(y, y_ref) <= F32_TOL


IMAGE_SHAPES = [  # small feature maps (a patch within 128 bytes of a plane): the input transform reads planes as they lie
    (1, 3, 4, 7, 7),      # 147 bytes: the last dwords of the tensor are fetched byte by byte
    (5, 70, 24, 7, 7),    # channels padded to 128, the last 58 zero
    (3, 200, 16, 5, 6),   # four ranges of 64 channels, planes of 30 bytes
    (9, 130, 8, 6, 6),    # one full 6x6 tile
    (520, 130, 8, 3, 2),  # ranges of 128 channels, the last half empty (Cin padded to 192)
    (2, 600, 8, 6, 6),    # more than 512 channels: the sums of M take four bytes, not three
    (3, 96, 8, 8, 8),     # 64 samples, four tiles per image in every form
    (2, 40, 8, 2, 16),    # one row of four 4x4 tiles (three 6x6 or 7x7 tiles)
    (3, 70, 8, 14, 14),   # 16, 9 or 4 tiles per image, patches of up to 121 bytes: two steps of 64
    (2, 64, 8, 9, 13),    # odd width
    (1, 20, 8, 16, 15),   # 16 tiles of 4x4; too wide for the 7x7 forms (generic kernel)
]


@pytest.mark.parametrize("alg", ALGS_STAGED)
@pytest.mark.parametrize("shape", IMAGE_SHAPES)
def test_small_images_taps_bit_exact(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 250 + len(alg) + sum(shape))
    print("case image", shape, alg, flush=True)
    xc, _, _, _ = uniform_case(shape, 350 + sum(shape))
    sx = oracle.calibrate_act_scales(xc // 2, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, sx=sx, sw=sw, return_taps=True)
    for name in ("V", "U", "M"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    assert rel_err(y, y_ref) <= F32_TOL
    if not alg.startswith("6x6") and -(-shape[1] // 64) in (1, 2, 4, 8):  # what the fused path takes
        y = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="fused", sx=sx, sw=sw)
        assert rel_err(y, y_ref) <= F32_TOL


@pytest.mark.parametrize("alg", ["7x7_p132", "4x4_p46"])
def test_staged_sums_at_the_three_byte_bound(binding, alg):
    """512 channels with every transform-domain operand at the clamp: sums of +-512 * 127^2 =
    +-8258048, the largest a three-byte sum of M has to hold, bit-exact."""
    shape = (2, 512, 20, 7, 7)
    rng = np.random.default_rng(77)
    x = rng.choice(np.array([-127, 127], dtype=np.int8), size=(shape[0], shape[1], shape[3], shape[4]))
    x[0] = 127  # a constant image: its zero-frequency point is at the clamp in every channel
    w = np.full((shape[2], shape[1], 3, 3), 127, dtype=np.int8)
    w[1::2] = -127
    print("case bound", alg, flush=True)
    sx = np.full_like(oracle.calibrate_act_scales(x, alg), 1e-3)
    sw = np.full_like(oracle.calibrate_filter_scales(w, alg), 1e-3)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, 0.02, 0.01, alg, return_taps=True)
    assert np.abs(taps_ref["M"]).max() == 512 * 127 * 127
    y, taps = binding.conv2d(x, w, 0.02, 0.01, mode="requant", alg=alg, sx=sx, sw=sw, return_taps=True)
    for name in ("V", "U", "M"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    assert rel_err(y, y_ref) <= F32_TOL


@pytest.mark.parametrize("bits", [4, 6])
@pytest.mark.parametrize("path", ["staged", "fused", "single"])
@pytest.mark.parametrize("alg", ["6x6_p88", "7x7_p144", "4x4_p46"])
def test_sub_int8_transform_domain(binding, alg, path, bits):
    """Transform-domain operands rounded to 4 or 6 bits (carried in int8 lanes), Sec. 6:
    taps bit-exact, output within tolerance, and the library's own abs-max calibration
    divides by the same bound as the oracle's."""
    import torch

    shape = (2, 24, 20, 14, 10)
    x, w, xs, ws = uniform_case(shape, 1100 + bits + len(alg))
    print("case bits", alg, path, bits, flush=True)
    qmax = 2 ** (bits - 1) - 1
    xc, _, _, _ = uniform_case(shape, 1200 + bits)
    sx = oracle.calibrate_act_scales(xc // 2, alg, qmax=qmax)
    sw = oracle.calibrate_filter_scales(w, alg, qmax=qmax)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, qmax=qmax, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path=path, sx=sx, sw=sw,
                             return_taps=True, transform_bits=bits)
    for name in taps:
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
        if name in ("V", "U"):
            assert np.abs(taps[name]).max() == qmax
    assert rel_err(y, y_ref) <= F32_TOL
    plan = binding.Plan(*shape, alg=alg, mode="requant", transform_bits=bits)
    wbuf = binding.device_buffer(plan.workspace_bytes)
    assert np.array_equal(plan.calibrate_act_scales(torch.from_numpy(xc // 2).cuda(), wbuf), sx)
    assert np.array_equal(plan.calibrate_filter_scales(torch.from_numpy(w).cuda(), wbuf), sw)
    plan.close()


@pytest.mark.parametrize("bits", [8, 6, 4])
def test_scale_granularity_ablation(binding, bits):
    """The granularity settings of Sec. 6's ablation (activations per tensor / per frequency,
    filters per channel / per channel and frequency) at int8, int6 and int4 in the transform
    domain, SFC-6(7x7,3x3): scales calibrated and grouped by the library, every setting bit-exact
    in its taps and within tolerance of the oracle; the error against direct convolution falls as
    the granularity gets finer (on synthetic data; accuracy itself needs ImageNet)."""
    import torch

    alg, shape = "7x7_p132", (4, 32, 24, 14, 14)
    d = synth.make_layer(synth.LayerShape("abl", *shape, "relu", True, 5))
    print("case ablation", bits, flush=True)
    qmax = 2 ** (bits - 1) - 1
    plan = binding.Plan(*shape, alg=alg, mode="requant", transform_bits=bits)
    wbuf = binding.device_buffer(plan.workspace_bytes)
    sx = plan.calibrate_act_scales(torch.from_numpy(d["x_calib"]).cuda(), wbuf)
    sw = plan.calibrate_filter_scales(torch.from_numpy(d["w"]).cuda(), wbuf)
    ref = oracle.dequantize(oracle.direct_conv(d["x"], d["w"]), d["x_scale"], d["w_scale"])
    errs = []
    for act, filt in (("tensor", "channel"), ("point", "channel"), ("point", "point"),
                      ("point", "channel_point")):
        gx, gw = plan.group_scales(sx, sw, act, filt)
        ox, ow = oracle.group_scales(oracle.calibrate_act_scales(d["x_calib"], alg, qmax=qmax),
                                     oracle.calibrate_filter_scales(d["w"], alg, qmax=qmax), act, filt)
        assert np.array_equal(gx, ox) and np.array_equal(gw, ow)
        y_ref, taps_ref = oracle.conv_requant(d["x"], d["w"], gx, gw, d["x_scale"], d["w_scale"], alg,
                                              qmax=qmax, return_taps=True)
        for path in ("staged", "fused"):
            y, taps = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg,
                                     path=path, sx=gx, sw=gw, return_taps=True, transform_bits=bits)
            for name in taps:
                assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), (name, act, filt)
            assert rel_err(y, y_ref) <= F32_TOL
        errs.append(float(np.sqrt(np.mean((y.astype(np.float64) - ref) ** 2))))
    plan.close()
    print("rms error vs direct convolution:", errs, flush=True)
    assert errs[0] > errs[1] > errs[3] and errs[2] > errs[3], errs


def test_single_filter_scale(binding):
    x, w, xs, _ = uniform_case((1, 16, 16, 32, 32), 7)
    ws = np.array([0.01], dtype=np.float32)
    acc = binding.conv2d(x, w, xs, ws, mode="exact", out="i32")
    assert np.array_equal(acc.astype(np.int64), oracle.direct_conv(x, w))
    y = binding.conv2d(x, w, xs, ws, mode="exact", out="f32")
    assert rel_err(y, oracle.dequantize(oracle.direct_conv(x, w), xs, ws)) <= F32_TOL


@pytest.mark.parametrize("alg", ALGS_STAGED)
def test_gpu_calibration_matches_oracle(binding, alg):
    import torch

    d = synth.make_layer(synth.LayerShape("cal", 4, 24, 20, 14, 10, "relu", True, 2))
    plan = binding.Plan(4, 24, 20, 14, 10, alg=alg, mode="requant")
    wbuf = binding.device_buffer(plan.workspace_bytes)
    xd = torch.from_numpy(d["x"]).cuda()
    wd = torch.from_numpy(d["w"]).cuda()
    sx = plan.calibrate_act_scales(xd, wbuf)
    sw = plan.calibrate_filter_scales(wd, wbuf)
    assert np.array_equal(sx, oracle.calibrate_act_scales(d["x"], alg))
    assert np.array_equal(sw, oracle.calibrate_filter_scales(d["w"], alg))
    # fewer calibration images than the plan's batch
    sx2 = plan.calibrate_act_scales(xd[:2].contiguous(), wbuf)
    assert np.array_equal(sx2, oracle.calibrate_act_scales(d["x"][:2], alg))
    plan.close()


# SFC-6(6x6,5x5) (Appendix A) and SFC-6(4x4,7x7) (Table 1): staged and fused paths
ALGS_5X5 = ["6x6_5x5_p184", "6x6_5x5_p196", "4x4_7x7_p184", "4x4_7x7_p196"]


@pytest.mark.parametrize("alg", ALGS_5X5)
@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_5x5_exact_mode_taps_and_sums_bit_exact(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 1300 + len(alg) + sum(shape), r=binding.KERNEL_SIZE[alg])
    print("case 5x5 exact", shape, alg, flush=True)
    acc_ref, taps_ref = oracle.conv_exact(x, w, alg, return_taps=True)
    assert np.array_equal(acc_ref, oracle.direct_conv(x, w))
    acc, taps = binding.conv2d(x, w, xs, ws, mode="exact", alg=alg, out="i32", return_taps=True)
    for name in ("V", "U", "M"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    assert np.array_equal(acc.astype(np.int64), acc_ref)
    y = binding.conv2d(x, w, xs, ws, mode="exact", alg=alg, out="f32")
    assert rel_err(y, oracle.dequantize(acc_ref, xs, ws)) <= F32_TOL


@pytest.mark.parametrize("alg", ALGS_5X5)
@pytest.mark.parametrize("shape", SMALL_SHAPES)
def test_5x5_requant_mode_taps_bit_exact_and_output_close(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 1400 + len(alg) + sum(shape), r=binding.KERNEL_SIZE[alg])
    print("case 5x5 requant", shape, alg, flush=True)
    xc, _, _, _ = uniform_case(shape, 1500 + sum(shape))
    sx = oracle.calibrate_act_scales(xc // 2, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, sx=sx, sw=sw, return_taps=True)
    for name in ("V", "U", "M"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    if x.size > 1:
        assert np.abs(taps["V"]).max() == 127  # the clamp was exercised
    assert rel_err(y, y_ref) <= F32_TOL


@pytest.mark.parametrize("alg", ALGS_5X5)
def test_5x5_calibration_int8_output_and_limits(binding, alg):
    """The library's abs-max calibration against the oracle's, the int8 + ReLU epilogue with
    4-bit and 8-bit transform domains on the staged and the fused path, and what the 5x5 forms
    do not take."""
    import torch

    shape = (4, 24, 20, 14, 10)
    d = synth.make_layer(synth.LayerShape("cal5", *shape, "relu", True, 2), kernel=binding.KERNEL_SIZE[alg])
    print("case 5x5 calibration", alg, flush=True)
    for bits in (8, 4):
        qmax = 2 ** (bits - 1) - 1
        plan = binding.Plan(*shape, alg=alg, mode="requant", transform_bits=bits)
        wbuf = binding.device_buffer(plan.workspace_bytes)
        sx = plan.calibrate_act_scales(torch.from_numpy(d["x_calib"]).cuda(), wbuf)
        sw = plan.calibrate_filter_scales(torch.from_numpy(d["w"]).cuda(), wbuf)
        plan.close()
        assert np.array_equal(sx, oracle.calibrate_act_scales(d["x_calib"], alg, qmax=qmax))
        assert np.array_equal(sw, oracle.calibrate_filter_scales(d["w"], alg, qmax=qmax))
        y_ref = oracle.conv_requant(d["x"], d["w"], sx, sw, d["x_scale"], d["w_scale"], alg, qmax=qmax)
        y = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg,
                           sx=sx, sw=sw, transform_bits=bits)
        assert rel_err(y, y_ref) <= F32_TOL
        y_scale = float(np.float32(max(y_ref.max(), 1e-6) / 127.0 * 0.8))
        for path in ("staged", "fused"):
            y8 = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg,
                                out="i8", path=path, sx=sx, sw=sw, y_scale=y_scale, transform_bits=bits)
            assert check_i8_against_oracle(y8, y_ref, y_scale) < 1e-3
    for kw in (dict(path="single"), dict(path="fused", Cin=330)):  # six 64-channel chunks
        args = dict(N=1, Cin=16, Cout=16, H=8, W=8, alg=alg)
        args.update(kw)
        with pytest.raises(binding.SfcError) as e:
            binding.Plan(**args)
        assert e.value.code == 2


@pytest.mark.parametrize("alg", ["6x6_5x5_p184", "4x4_7x7_p184"])
def test_5x5_full_size_against_oracle(binding, alg):
    """A 5x5 (7x7) layer on the resnet28 geometry (128 -> 128 channels, 28x28, 64 images): every
    tap and every output element against the oracle, and the exact mode against direct
    convolution (7x7 filters: on the first 64 input channels, the range exact mode guarantees)."""
    shape = synth.LAYERS["resnet28"]
    print("case 5x5 full", alg, flush=True)
    d = synth.make_layer(shape, kernel=binding.KERNEL_SIZE[alg])
    sx = oracle.calibrate_act_scales(d["x_calib"], alg)
    sw = oracle.calibrate_filter_scales(d["w"], alg)
    y_ref, taps_ref = oracle.conv_requant(d["x"], d["w"], sx, sw, d["x_scale"], d["w_scale"], alg,
                                          return_taps=True)
    y, taps = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg,
                             sx=sx, sw=sw, return_taps=True)
    for tap in ("V", "U", "M"):
        assert np.array_equal(taps[tap].astype(np.int64), taps_ref[tap]), tap
    assert rel_err(y, y_ref) <= F32_TOL
    yf, taps = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg,
                              path="fused", sx=sx, sw=sw, return_taps=True)
    assert np.array_equal(taps["V"].astype(np.int64), taps_ref["V"])
    assert rel_err(yf, y_ref) <= F32_TOL
    xe, we = d["x"], d["w"]
    if binding.KERNEL_SIZE[alg] == 7:
        xe, we = np.ascontiguousarray(xe[:16, :64]), np.ascontiguousarray(we[:, :64])
    acc = binding.conv2d(xe, we, d["x_scale"], d["w_scale"], mode="exact", alg=alg, out="i32")
    assert np.array_equal(acc.astype(np.int64), oracle.direct_conv(xe, we))


WIDE_SHAPES = [  # rows too wide for whole-strip staging in the generic input kernel
    (1, 3, 4, 9, 300),    # odd tile count per row, W a multiple of 4
    (2, 5, 3, 13, 1024),  # the widest row the library takes
    (1, 70, 8, 7, 203),   # two channel slices, W not a multiple of 4
]


@pytest.mark.parametrize("alg", ["6x6_p88", "7x7_p144", "4x4_p46", "6x6_5x5_p184", "4x4_7x7_p196"])
@pytest.mark.parametrize("shape", WIDE_SHAPES)
def test_wide_rows_exact_calibration_and_requant(binding, shape, alg):
    import torch

    r = binding.KERNEL_SIZE[alg]
    x, w, xs, ws = uniform_case(shape, 1800 + len(alg) + sum(shape), r=r)
    print("case wide", shape, alg, flush=True)
    acc_ref, taps_ref = oracle.conv_exact(x, w, alg, return_taps=True)
    acc, taps = binding.conv2d(x, w, xs, ws, mode="exact", alg=alg, out="i32", return_taps=True)
    assert np.array_equal(taps["V"].astype(np.int64), taps_ref["V"])
    assert np.array_equal(acc.astype(np.int64), acc_ref)
    plan = binding.Plan(*shape, alg=alg, mode="requant")
    wbuf = binding.device_buffer(plan.workspace_bytes)
    sx = plan.calibrate_act_scales(torch.from_numpy(x // 2).cuda(), wbuf)
    plan.close()
    assert np.array_equal(sx, oracle.calibrate_act_scales(x // 2, alg))
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, sx=sx, sw=sw, return_taps=True)
    for name in ("V", "U", "M"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    assert rel_err(y, y_ref) <= F32_TOL


FULL = ["resnet56", "resnet28", "resnet14", "resnet7"]


@pytest.mark.parametrize("alg", ["4x4_p46", "4x4_p49"])
def test_sfc4_full_size_and_int8_output(binding, alg):
    """SFC-4(4x4,3x3) on resnet28 (4x4 tiles divide 28): every tap and output element; then the
    int8 + ReLU epilogue on the staged and fused paths."""
    shape = synth.LAYERS["resnet28"]
    print("case sfc4 full", alg, flush=True)
    d = synth.make_layer(shape)
    sx = oracle.calibrate_act_scales(d["x_calib"], alg)
    sw = oracle.calibrate_filter_scales(d["w"], alg)
    y_ref, taps_ref = oracle.conv_requant(d["x"], d["w"], sx, sw, d["x_scale"], d["w_scale"], alg,
                                          return_taps=True)
    y, taps = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg,
                             sx=sx, sw=sw, return_taps=True)
    for tap in ("V", "U", "M"):
        assert np.array_equal(taps[tap].astype(np.int64), taps_ref[tap]), tap
    assert rel_err(y, y_ref) <= F32_TOL
    y_scale = float(np.float32(max(y_ref.max(), 1e-6) / 127.0 * 0.8))
    for path in ("staged", "fused"):
        y8 = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg, out="i8",
                            path=path, sx=sx, sw=sw, y_scale=y_scale)
        assert check_i8_against_oracle(y8, y_ref, y_scale) < 1e-3


@pytest.mark.parametrize("name,alg", [(n, "6x6_p88") for n in FULL] +
                         [("resnet14", "7x7_p132"), ("resnet7", "7x7_p132"),  # the 7x7 stretch of Sec. 4.2
                          ("resnet14", "4x4_p46"), ("resnet7", "4x4_p46")])   # ragged 4x4 tiles
def test_full_size_requant_against_oracle(binding, name, alg):
    """The ResNet-shaped workloads at full size, staged path: every element of V, U, M and y."""
    shape = synth.LAYERS[name]
    print("case full", name, alg, flush=True)
    d = synth.make_layer(shape)
    sx = oracle.calibrate_act_scales(d["x_calib"], alg)
    sw = oracle.calibrate_filter_scales(d["w"], alg)
    y_ref, taps_ref = oracle.conv_requant(d["x"], d["w"], sx, sw, d["x_scale"], d["w_scale"], alg,
                                          return_taps=True)
    y, taps = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg, sx=sx,
                             sw=sw, return_taps=True)
    for tap in ("V", "U", "M"):
        assert np.array_equal(taps[tap].astype(np.int64), taps_ref[tap]), tap
    assert rel_err(y, y_ref) <= F32_TOL
    # the approximation itself stays close to the direct convolution
    direct = oracle.dequantize(oracle.direct_conv(d["x"], d["w"]), d["x_scale"], d["w_scale"])
    rms = np.sqrt(np.mean((y - direct) ** 2)) / np.sqrt(np.mean(direct**2))
    assert rms < 0.05


@pytest.mark.parametrize("name", ["resnet56", "resnet7"])
def test_full_size_exact_against_direct_conv(binding, name):
    shape = synth.LAYERS[name]
    print("case full exact", name, flush=True)
    d = synth.make_layer(shape)
    ref = oracle.direct_conv(d["x"], d["w"])
    assert np.abs(ref).max() * 36 < 2**31  # int32 sums hold for this data (Cin = 512 included)
    # beyond 404 channels the caller vouches for the 32-bit sums (checked on this data above)
    flags = binding.FLAG_EXACT_WIDE if shape.Cin > 404 else 0
    acc = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="exact", out="i32", flags=flags)
    assert np.array_equal(acc.astype(np.int64), ref)


# ---- fused path: products never leave the chip, so only V, U and y can be compared ----

FUSED_SHAPES = [
    (1, 16, 16, 32, 32),
    (2, 3, 5, 14, 14),
    (1, 4, 4, 7, 7),  # odd W: scalar stores
    (2, 2, 3, 13, 9),
    (1, 1, 1, 1, 1),
    (3, 70, 40, 9, 20),  # two 64-channel chunks, Cout 40: a partly idle wave
    (5, 64, 64, 12, 18),  # 30 tiles: padding rows in the last block
    (2, 200, 72, 11, 7),  # four chunks (Cin padded to 256), two workgroups along Cout
    (1, 500, 24, 8, 8),  # eight chunks
    (3, 460, 72, 14, 14),  # eight chunks, three filter pairs of 32, whole-image stores with 7x7 tiles
    (2, 512, 40, 9, 13),  # eight chunks, odd W
    # small feature maps, staged as whole images: batch not a multiple of the images per
    # workgroup, plane sizes that are / are not whole dwords, planes above 64 dwords
    (5, 20, 8, 7, 7),
    (3, 9, 8, 14, 14),
    (7, 3, 4, 12, 12),
    (2, 70, 16, 28, 28),
]


@pytest.mark.parametrize("alg", ALGS_STAGED)
@pytest.mark.parametrize("shape", FUSED_SHAPES)
def test_fused_path_matches_oracle(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 400 + len(alg) + sum(shape))
    print("case fused", shape, alg, flush=True)
    xc, _, _, _ = uniform_case(shape, 500 + sum(shape))
    sx = oracle.calibrate_act_scales(xc // 2, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="fused", sx=sx, sw=sw,
                             return_taps=True)
    for name in ("V", "U"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    assert rel_err(y, y_ref) <= F32_TOL
    # and it agrees with the staged path of the same library to float32 rounding
    y_staged = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="staged", sx=sx, sw=sw)
    assert rel_err(y, y_staged.astype(np.float64)) <= F32_TOL


@pytest.mark.parametrize("alg", ALGS_5X5)
@pytest.mark.parametrize("shape", FUSED_SHAPES)
def test_5x5_fused_path_matches_oracle(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 1600 + len(alg) + sum(shape), r=binding.KERNEL_SIZE[alg])
    print("case 5x5 fused", shape, alg, flush=True)
    xc, _, _, _ = uniform_case(shape, 1700 + sum(shape))
    sx = oracle.calibrate_act_scales(xc // 2, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="fused", sx=sx, sw=sw,
                             return_taps=True)
    for name in ("V", "U"):
        assert np.array_equal(taps[name].astype(np.int64), taps_ref[name]), name
    assert rel_err(y, y_ref) <= F32_TOL


SINGLE_SHAPES = [
    (1, 16, 16, 32, 32),
    (2, 3, 5, 14, 14),
    (1, 4, 4, 7, 7),  # odd W: scalar stores
    (2, 2, 3, 13, 9),
    (1, 1, 1, 1, 1),
    (3, 60, 40, 9, 20),
    (5, 64, 64, 12, 18),
    (2, 64, 72, 11, 7),  # two filter groups
    (20, 7, 130, 7, 7),  # many strips per workgroup, three filter groups
    (1, 33, 17, 56, 56),  # two tile-column chunks per strip
    (2, 5, 9, 6, 61),  # wide and flat: chunks of nine or eight tile columns
    (5, 20, 8, 7, 7),  # whole-image staging, see FUSED_SHAPES
    (3, 9, 8, 14, 14),
    (7, 3, 4, 12, 12),
    (2, 64, 16, 28, 28),
]


@pytest.mark.parametrize("alg", ALGS_STAGED)
@pytest.mark.parametrize("shape", SINGLE_SHAPES)
def test_single_kernel_path_matches_oracle(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 700 + len(alg) + sum(shape))
    print("case single", shape, alg, flush=True)
    xc, _, _, _ = uniform_case(shape, 800 + sum(shape))
    sx = oracle.calibrate_act_scales(xc // 2, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="single", sx=sx, sw=sw,
                             return_taps=True)
    assert np.array_equal(taps["U"].astype(np.int64), taps_ref["U"])
    assert rel_err(y, y_ref) <= F32_TOL


SINGLE_WIDE_SHAPES = [  # two 64-channel chunks in one kernel (the SFC-4 forms)
    (3, 70, 40, 9, 20),
    (2, 128, 136, 11, 7),   # nine groups of 16 filters: two workgroups along Cout, odd W
    (1, 100, 24, 28, 28),   # rectangles of two strips
    (2, 128, 16, 14, 14),   # whole-image staging
    (5, 65, 8, 7, 7),
    (1, 96, 130, 56, 56),   # one strip per workgroup
    (2, 127, 5, 6, 61),
]


@pytest.mark.parametrize("alg", ["4x4_p46", "4x4_p49"])
@pytest.mark.parametrize("shape", SINGLE_WIDE_SHAPES)
def test_single_kernel_path_with_two_channel_chunks(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 750 + len(alg) + sum(shape))
    print("case single wide", shape, alg, flush=True)
    xc, _, _, _ = uniform_case(shape, 850 + sum(shape))
    sx = oracle.calibrate_act_scales(xc // 2, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="single", sx=sx, sw=sw,
                             return_taps=True)
    assert np.array_equal(taps["U"].astype(np.int64), taps_ref["U"])
    assert rel_err(y, y_ref) <= F32_TOL
    y_scale = float(np.float32(max(y_ref.max(), 1e-6) / 127.0 * 0.8))
    y8 = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="single", out="i8", sx=sx, sw=sw,
                        y_scale=y_scale)
    assert check_i8_against_oracle(y8, y_ref, y_scale) < 1e-3


def test_single_kernel_path_channel_limits(binding):
    with pytest.raises(binding.SfcError) as e:
        binding.Plan(1, 65, 16, 8, 8, path="single")  # 6x6 tiles: one chunk of 64 channels
    assert e.value.code == 2
    for shape in ((1, 129, 16, 28, 28),   # SFC-4: two chunks on maps of more than 16 tiles ...
                  (1, 513, 16, 8, 8)):    # ... eight chunks on smaller ones
        with pytest.raises(binding.SfcError) as e:
            binding.Plan(*shape, alg="4x4_p46", path="single")
        assert e.value.code == 2


@pytest.mark.parametrize("name,alg", [("resnet56", a) for a in ("6x6_p88", "7x7_p132", "4x4_p46", "4x4_p49")] +
                         [("resnet28", "4x4_p46"), ("resnet28", "4x4_p49")])
def test_full_size_single_kernel_against_oracle(binding, name, alg):
    """resnet56 and resnet28 in the launch configuration bench.py times, every output element."""
    shape = synth.LAYERS[name]
    print("case full single", name, alg, flush=True)
    d = synth.make_layer(shape)
    sx = oracle.calibrate_act_scales(d["x_calib"], alg)
    sw = oracle.calibrate_filter_scales(d["w"], alg)
    y_ref = oracle.conv_requant(d["x"], d["w"], sx, sw, d["x_scale"], d["w_scale"], alg)
    y = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg, path="single",
                       sx=sx, sw=sw)
    assert rel_err(y, y_ref) <= F32_TOL


def test_fused_path_rejects_unsupported_channel_counts(binding):
    with pytest.raises(binding.SfcError) as e:
        binding.Plan(1, 3 * 64, 16, 8, 8, path="fused")  # three chunks
    assert e.value.code == 2


@pytest.mark.parametrize("alg", ["6x6_p88", "7x7_p132", "4x4_p46"])
@pytest.mark.parametrize("name", FULL)
def test_full_size_fused_against_oracle(binding, name, alg):
    """The launch configuration bench.py times, every output element (V as well)."""
    shape = synth.LAYERS[name]
    print("case full fused", name, alg, flush=True)
    d = synth.make_layer(shape)
    sx = oracle.calibrate_act_scales(d["x_calib"], alg)
    sw = oracle.calibrate_filter_scales(d["w"], alg)
    y_ref, taps_ref = oracle.conv_requant(d["x"], d["w"], sx, sw, d["x_scale"], d["w_scale"], alg,
                                          return_taps=True)
    y, taps = binding.conv2d(d["x"], d["w"], d["x_scale"], d["w_scale"], mode="requant", alg=alg,
                             path="fused", sx=sx, sw=sw, return_taps=True)
    assert np.array_equal(taps["V"].astype(np.int64), taps_ref["V"])
    assert rel_err(y, y_ref) <= F32_TOL


# ---- int8 + ReLU epilogue (chaining stride-1 layers of a stack) ----------------------


def check_i8_against_oracle(y8, y_ref, y_scale):
    """Exact wherever the oracle's value is not within float32 reach of a rounding boundary."""
    inv = float(oracle.reciprocal_f32(y_scale))
    t = np.maximum(y_ref, 0.0) * inv
    q_ref = np.clip(np.rint(t), 0, 127)
    assert np.array_equal(q_ref.astype(np.int8), oracle.requantize_activation(y_ref, y_scale))
    diff = y8.astype(np.int64) - q_ref.astype(np.int64)
    slack = F32_TOL * np.abs(y_ref).max() * inv + 1e-6
    near_boundary = np.abs(t - np.floor(t) - 0.5) <= slack
    assert np.abs(diff).max() <= 1
    assert np.all(diff[~near_boundary] == 0)
    return float(np.count_nonzero(diff)) / diff.size


@pytest.mark.parametrize("alg", ["6x6_p88", "4x4_p46"])
@pytest.mark.parametrize("path", ["staged", "fused", "single"])
@pytest.mark.parametrize("shape", [(1, 16, 16, 32, 32), (2, 3, 5, 14, 14), (1, 4, 4, 7, 7), (3, 70, 40, 9, 20)])
def test_int8_relu_output(binding, shape, path, alg):
    if path == "single" and shape[1] > 64:
        shape = (shape[0], 50, *shape[2:])
    x, w, xs, ws = uniform_case(shape, 600 + sum(shape))
    print("case i8", shape, path, alg, flush=True)
    sx = oracle.calibrate_act_scales(x, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg)
    y_scale = float(np.float32(max(y_ref.max(), 1e-6) / 127.0 * 0.8))  # 0.8: some values clamp at 127
    y8 = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path=path, out="i8", sx=sx, sw=sw,
                        y_scale=y_scale)
    assert y8.dtype == np.int8 and y8.min() == 0 and y8.max() == 127
    frac = check_i8_against_oracle(y8, y_ref, y_scale)
    assert frac < 1e-3


@pytest.mark.parametrize("alg", ["7x7_p132", "7x7_p144", "4x4_p46", "4x4_p49"])
@pytest.mark.parametrize("path", ["staged", "fused"])
@pytest.mark.parametrize("case", [  # (N, Cin, Cout, tile rows, tile columns)
    (1, 4, 4, 1, 1),      # one tile, one filter quad
    (37, 20, 44, 1, 1),   # ragged last 16-tile block, filters end inside a filter group
    (16, 64, 96, 1, 1),   # whole blocks and groups
    (5, 9, 6, 1, 1),      # Cout not a multiple of 4: row-by-row stores
    (2, 5, 12, 1, 2),     # two tiles per image
    (3, 100, 8, 2, 2),    # four tiles per image, two 64-channel slices
    (3, 4, 8, 2, 4),      # eight tiles per image: 24 tiles, a ragged second block
    (2, 16, 36, 4, 4),    # sixteen tiles per image: one image per wave
])
def test_feature_maps_of_whole_images_per_wave(binding, case, path, alg):
    """7x7 or 4x4 tiles that cover the map exactly, 1, 2, 4, 8 or 16 to an image: the output
    transform writes whole planes of y.  float32 and int8 outputs against the oracle."""
    m = oracle.tile_out(alg)
    shape = (*case[:3], m * case[3], m * case[4])
    x, w, xs, ws = uniform_case(shape, 650 + sum(shape))
    print("case planes", shape, path, alg, flush=True)
    sx = oracle.calibrate_act_scales(x, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg)
    y = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path=path, sx=sx, sw=sw)
    assert y.shape == y_ref.shape
    assert rel_err(y, y_ref) <= F32_TOL
    y_scale = float(np.float32(max(y_ref.max(), 1e-6) / 127.0 * 0.8))
    y8 = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path=path, out="i8", sx=sx,
                        sw=sw, y_scale=y_scale)
    assert y8.dtype == np.int8 and y8.min() == 0 and y8.max() == 127
    assert check_i8_against_oracle(y8, y_ref, y_scale) < 1e-3


def test_int8_output_needs_its_scale(binding):
    import torch

    plan = binding.Plan(1, 16, 16, 8, 8, out="i8", path="fused")
    with pytest.raises(binding.SfcError) as e:
        binding.Plan(1, 16, 16, 8, 8, out="i8", mode="exact")
    assert e.value.code == 2
    p = plan.P
    plan.set_point_scales(np.ones(p, np.float32), np.ones((p, 16), np.float32))
    w = torch.zeros((16, 16, 3, 3), dtype=torch.int8, device="cuda")
    fbuf = binding.device_buffer(plan.filter_bytes)
    plan.transform_filter(w, np.ones(16, np.float32), fbuf)
    x = torch.zeros((1, 16, 8, 8), dtype=torch.int8, device="cuda")
    y = torch.zeros((1, 16, 8, 8), dtype=torch.int8, device="cuda")
    ws = binding.device_buffer(plan.workspace_bytes)
    with pytest.raises(binding.SfcError) as e:
        plan.conv2d(x, 0.02, y, ws)
    assert e.value.code == 4
    plan.set_output_scale(0.5)
    plan.conv2d(x, 0.02, y, ws)
    torch.cuda.synchronize()
    plan.close()


def test_resnet18_shaped_stack_chained_with_int8_activations(binding):
    """The 13 stride-1 3x3 layers at batch 64 exactly as bench.py runs them: layers built by
    ``layers.Layer`` (algorithm and path chosen by the library, the library's own abs-max
    calibration, int8 + ReLU output with the same output scale), chained inside each resolution
    stage.

    Every layer is checked against the oracle on the oracle's own input of that layer, with the
    scales the library calibrated (the scales are inputs of both sides; that the library's
    calibration equals the oracle's is test_gpu_calibration_matches_oracle); the library's
    self-chained run must then stay close to the oracle's chain."""
    from paper_2407_02913_amd import layers

    x_ref = x_gpu = None
    prev = None
    for idx, shape in enumerate(synth.stack_layers()):
        assert shape.N == synth.STACK_BATCH == 64
        d = synth.make_layer(shape, batch=4)  # weights, filter scales, calibration activations
        layer = layers.Layer(shape, d, out="i8", alg="auto", path="auto")
        print("case stack layer", idx, shape.name, layer.alg, layer.path, flush=True)
        if prev is None or (shape.Cin, shape.H) != (prev.Cin, prev.H):
            rng = np.random.default_rng(synth.BASE_SEED + shape.Cin)
            x_ref = x_gpu = synth.activations((shape.N, shape.Cin, shape.H, shape.W), "relu", rng)
        y_ref = oracle.conv_requant(x_ref, d["w"], layer.sx, layer.sw, d["x_scale"], d["w_scale"], layer.alg)
        y8 = layers.np_conv(layer, x_ref)
        frac = check_i8_against_oracle(y8, y_ref, layer.y_scale)
        assert frac < 1e-3
        assert y8.max() >= 32  # the output scale puts the activations into the int8 range
        # self-chained: the library's own previous output is this layer's input
        y8_chain = layers.np_conv(layer, x_gpu)
        x_next_ref = oracle.requantize_activation(y_ref, layer.y_scale)
        # (a sanity check of the chain, not the parity bar: single steps of difference at
        # rounding boundaries of one layer spread through the next ones of the stage)
        delta = np.abs(y8_chain.astype(np.int64) - x_next_ref.astype(np.int64))
        assert delta.max() <= 4 and np.mean(delta != 0) < 0.01
        x_ref, x_gpu, prev = x_next_ref, y8_chain, shape
        layer.close()


@pytest.mark.parametrize("name", FULL)
def test_single_layers_as_benchmarked(binding, name):
    """The four ResNet-shaped layers exactly as bench.py runs them (``layers.Layer``: algorithm
    and path chosen by the library, its own calibration, float32 output), every element."""
    from paper_2407_02913_amd import layers

    shape = synth.LAYERS[name]
    d = synth.make_layer(shape)
    layer = layers.Layer(shape, d, out="f32", alg="auto", path="auto")
    print("case layer as benchmarked", name, layer.alg, layer.path, flush=True)
    assert np.array_equal(layer.sx, oracle.calibrate_act_scales(d["x_calib"], layer.alg))
    assert np.array_equal(layer.sw, oracle.calibrate_filter_scales(d["w"], layer.alg))
    y_ref = oracle.conv_requant(d["x"], d["w"], layer.sx, layer.sw, d["x_scale"], d["w_scale"], layer.alg)
    y = layers.np_conv(layer, d["x"])
    assert rel_err(y, y_ref) <= F32_TOL
    layer.close()


SINGLE_DEEP_SHAPES = [  # 256 / 512 input channels on small maps: products accumulated chunk by chunk
    (3, 256, 72, 14, 14),   # one image (16 tiles) per workgroup, two workgroups along Cout
    (5, 200, 64, 7, 7),     # four images per workgroup, ragged last group; four chunks, the last part empty
    (2, 512, 40, 8, 8),     # eight chunks
    (9, 300, 130, 4, 4),    # one tile per image: 16 images per workgroup; five chunks
    (1, 256, 16, 13, 9),    # odd W: single-element stores
    (2, 512, 512, 7, 7),
]


@pytest.mark.parametrize("alg", ["4x4_p46", "4x4_p49"])
@pytest.mark.parametrize("shape", SINGLE_DEEP_SHAPES)
def test_single_kernel_path_with_many_channel_chunks(binding, shape, alg):
    x, w, xs, ws = uniform_case(shape, 770 + len(alg) + sum(shape))
    print("case single deep", shape, alg, flush=True)
    xc, _, _, _ = uniform_case(shape, 870 + sum(shape))
    sx = oracle.calibrate_act_scales(xc // 2, alg)
    sw = oracle.calibrate_filter_scales(w, alg)
    y_ref, taps_ref = oracle.conv_requant(x, w, sx, sw, xs, ws, alg, return_taps=True)
    y, taps = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="single", sx=sx, sw=sw,
                             return_taps=True)
    assert np.array_equal(taps["U"].astype(np.int64), taps_ref["U"])
    assert rel_err(y, y_ref) <= F32_TOL
    y_scale = float(np.float32(max(y_ref.max(), 1e-6) / 127.0 * 0.8))
    y8 = binding.conv2d(x, w, xs, ws, mode="requant", alg=alg, path="single", out="i8", sx=sx, sw=sw,
                        y_scale=y_scale)
    assert check_i8_against_oracle(y8, y_ref, y_scale) < 1e-3
    # larger maps do not fit: the path is refused
    with pytest.raises(binding.SfcError) as e:
        binding.Plan(1, shape[1], 16, 28, 28, alg=alg, path="single")
    assert e.value.code == 2
