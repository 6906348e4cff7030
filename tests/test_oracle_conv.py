"""Pins for the CPU oracle's convolution (run without a GPU).

Each test checks the oracle against something other than itself: exact rational
brute force of Eq. (1) ("The Convolution Operator"), the impulse-response closed
form, a library dense convolution for the all-ones mask, and invariants that a
dropped term, wrong sign/index or transposed operand would break.
"""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from pconv_inputs import PATTERN_TABLE, LayerSpec, make_input, make_layer


def bit(mask, r, s):
    return (int(mask) >> (3 * r + s)) & 1


def brute_force(x, w, pid, conn, table, bias, stride, pad, relu):
    """Eq. (1) transcribed literally in exact rational arithmetic (NCHW)."""
    n_img, c_in, h, wd = x.shape
    c_out = w.shape[0]
    ho = (h + 2 * pad - 3) // stride + 1
    wo = (wd + 2 * pad - 3) // stride + 1
    y = np.empty((n_img, c_out, ho, wo), dtype=object)
    sc = np.empty((n_img, c_out, ho, wo), dtype=object)
    for n in range(n_img):
        for f in range(c_out):
            for oy in range(ho):
                for ox in range(wo):
                    acc = Fraction(float(bias[f])) if bias is not None else Fraction(0)
                    sab = abs(acc)
                    for c in range(c_in):
                        if not conn[f, c]:
                            continue
                        for r in range(3):
                            for s in range(3):
                                if not bit(table[pid[f, c]], r, s):
                                    continue
                                iy, ix = oy * stride + r - pad, ox * stride + s - pad
                                if 0 <= iy < h and 0 <= ix < wd:
                                    p = Fraction(float(w[f, c, r, s])) * Fraction(float(x[n, c, iy, ix]))
                                    acc += p
                                    sab += abs(p)
                    y[n, f, oy, ox] = max(acc, Fraction(0)) if relu else acc
                    sc[n, f, oy, ox] = sab
    return y, sc


def tiny(c_in, c_out, h, w, n=1, seed=0, stride=1, keep_div=2.0, patterns=8):
    spec = LayerSpec("tiny", n, c_in, c_out, h, w, stride=stride, num_patterns=patterns,
                     pattern_dist="uniform", keep_div=keep_div, count_dist="bernoulli")
    layer = make_layer(spec, seed)
    x = make_input(spec, seed)
    x -= 0.3   # make some activations negative so |.| in S matters
    return spec, layer, x


@pytest.mark.parametrize("stride", [1, 2])
@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("shape", [(2, 3, 5, 5), (3, 2, 4, 7), (1, 1, 3, 3), (2, 2, 6, 5)])
def test_brute_force_exact(shape, stride, relu):
    c_in, c_out, h, w = shape
    spec, L, x = tiny(c_in, c_out, h, w, n=2, seed=11 + h, stride=stride)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    y, s = oracle.conv2d(x, wt, L["bias"], stride=stride, pad=1, relu=relu)
    yb, sb = brute_force(x, L["w"], L["pattern_id"], L["conn"], L["table"], L["bias"],
                         stride, 1, relu)
    yb = np.array([[float(v) for v in row] for row in yb.reshape(-1, 1)]).reshape(y.shape)
    sbf = np.array([[float(v) for v in row] for row in sb.reshape(-1, 1)]).reshape(y.shape)
    # fp64 accumulation of <= 9*c_in products: error far below 1e-13 * S
    assert np.all(np.abs(y - yb) <= 1e-13 * sbf + 1e-300)
    assert np.all(np.abs(s - sbf) <= 1e-13 * sbf + 1e-300)


def test_config1_brute_force_sample():
    """Config 1 (16->16 @16x16): sampled outputs against the exact brute force."""
    from pconv_inputs import base_seed, config_layers
    spec = config_layers(1)[0]
    L = make_layer(spec, base_seed(1)); x = make_input(spec, base_seed(1))
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    y, s = oracle.conv2d(x, wt, L["bias"])
    sub = slice(0, 1), slice(0, 16), slice(0, 16), slice(0, 16)
    yb, _ = brute_force(x[:, :, :6, :6], L["w"], L["pattern_id"], L["conn"], L["table"],
                        L["bias"], 1, 1, False)
    # interior of the cropped image (rows/cols 0..4) sees the same neighbourhood
    for f in range(16):
        for oy in range(5):
            for ox in range(5):
                assert abs(y[0, f, oy, ox] - float(yb[0, f, oy, ox])) <= 1e-13 * s[0, f, oy, ox]


@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
def test_impulse_reads_masked_weights_back(layout):
    """X = unit impulse at (c0,y0,x0)  =>  Y[f,y,x] = W~[f,c0,y0-y+1,x0-x+1] (stride 1)."""
    spec, L, _ = tiny(4, 5, 7, 6, seed=3)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    c0, y0, x0 = 2, 3, 4
    x = np.zeros((1, 4, 7, 6), np.float32)
    x[0, c0, y0, x0] = 1.0
    xin = x if layout == "nchw" else np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    y, _ = oracle.conv2d(xin, wt, None, layout=layout)
    if layout == "nhwc":
        y = y.transpose(0, 3, 1, 2)
    expect = np.zeros_like(y)
    mask = L["table"][L["pattern_id"]]
    for f in range(5):
        for r in range(3):
            for s in range(3):
                oy, ox = y0 - r + 1, x0 - s + 1
                if 0 <= oy < 7 and 0 <= ox < 6 and L["conn"][f, c0] and bit(mask[f, c0], r, s):
                    expect[0, f, oy, ox] = np.float64(L["w"][f, c0, r, s])
    assert np.array_equal(y, expect)
    assert np.count_nonzero(expect) > 0


@pytest.mark.parametrize("stride", [1, 2])
def test_all_ones_mask_is_dense_conv(stride):
    """Mask 0x1FF and full connectivity reduce to the textbook dense convolution."""
    rng = np.random.default_rng(5)
    w = rng.standard_normal((6, 5, 3, 3)).astype(np.float32)
    x = rng.standard_normal((2, 5, 9, 8)).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    table = np.array([0x1FF], np.uint16)
    pid = np.zeros((6, 5), np.uint8); conn = np.ones((6, 5), np.uint8)
    wt = oracle.masked_weights(w, pid, conn, table)
    y, s = oracle.conv2d(x, wt, b, stride=stride)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     torch.from_numpy(b).double(), stride=stride, padding=1).numpy()
    assert np.allclose(y, ref, rtol=0, atol=1e-12)
    sref = torch.nn.functional.conv2d(torch.from_numpy(x).double().abs(),
                                      torch.from_numpy(w).double().abs(),
                                      torch.from_numpy(b).double().abs(), stride=stride,
                                      padding=1).numpy()
    assert np.allclose(s, sref, rtol=1e-13, atol=0)


def test_masked_equals_library_conv_of_masked_weights():
    """General masks: oracle == library dense conv over independently masked weights."""
    spec, L, x = tiny(7, 9, 11, 10, n=2, seed=21, patterns=12)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    wm = np.zeros_like(L["w"], dtype=np.float64)
    for f in range(9):
        for c in range(7):
            if L["conn"][f, c]:
                m = int(L["table"][L["pattern_id"][f, c]])
                for t in range(9):
                    if (m >> t) & 1:
                        wm[f, c, t // 3, t % 3] = L["w"][f, c, t // 3, t % 3]
    assert np.array_equal(wt, wm)
    y, _ = oracle.conv2d(x, wt, L["bias"], relu=True)
    ref = torch.relu(torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(wm),
                                                torch.from_numpy(L["bias"]).double(), padding=1))
    assert np.allclose(y, ref.numpy(), rtol=0, atol=1e-12)


def test_zeroed_kernel_contributes_exactly_its_dense_part():
    spec, L, x = tiny(5, 4, 8, 8, seed=9)
    f0, c0 = 1, 2
    conn_on = L["conn"].copy(); conn_on[f0, c0] = 1
    conn_off = conn_on.copy(); conn_off[f0, c0] = 0
    w_on = oracle.masked_weights(L["w"], L["pattern_id"], conn_on, L["table"])
    w_off = oracle.masked_weights(L["w"], L["pattern_id"], conn_off, L["table"])
    y_on, _ = oracle.conv2d(x, w_on, None)
    y_off, _ = oracle.conv2d(x, w_off, None)
    delta = y_on - y_off
    k = torch.from_numpy(w_on[f0:f0 + 1, c0:c0 + 1])
    part = torch.nn.functional.conv2d(torch.from_numpy(x[:, c0:c0 + 1]).double(), k, padding=1).numpy()
    assert np.allclose(delta[:, f0], part[:, 0], atol=1e-12)
    others = [f for f in range(4) if f != f0]
    assert np.array_equal(y_on[:, others], y_off[:, others])
    assert np.any(delta[:, f0] != 0)


def test_pattern_split_linearity():
    """sum_p conv(W (.) [pattern == p]) == conv(W)."""
    spec, L, x = tiny(6, 5, 9, 9, seed=13)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    y, _ = oracle.conv2d(x, wt, None)
    total = np.zeros_like(y)
    for p in range(len(L["table"])):
        conn_p = (L["conn"] != 0) & (L["pattern_id"] == p)
        wp = oracle.masked_weights(L["w"], L["pattern_id"], conn_p.astype(np.uint8), L["table"])
        total += oracle.conv2d(x, wp, None)[0]
    assert np.allclose(total, y, atol=1e-12)


def test_constant_input_interior_and_shift():
    spec, L, _ = tiny(4, 3, 9, 9, seed=2)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    x = np.full((1, 4, 9, 9), 2.0, np.float32)
    y, _ = oracle.conv2d(x, wt, L["bias"])
    expect = L["bias"].astype(np.float64) + 2.0 * wt.sum(axis=(1, 2, 3))
    assert np.allclose(y[0, :, 1:-1, 1:-1], expect[:, None, None], atol=1e-12)
    # shift equivariance in the interior
    rng = np.random.default_rng(4)
    x = np.zeros((1, 4, 12, 12), np.float32)
    x[:, :, 3:7, 3:7] = rng.standard_normal((1, 4, 4, 4))
    xs = np.roll(x, (2, 3), axis=(2, 3))
    y0, _ = oracle.conv2d(x, wt, None); y1, _ = oracle.conv2d(xs, wt, None)
    assert np.array_equal(np.roll(y0, (2, 3), axis=(2, 3)), y1)


def test_stride2_is_subsampled_stride1():
    for (h, w) in [(8, 8), (7, 9)]:
        spec, L, x = tiny(3, 4, h, w, seed=h)
        wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
        y1, s1 = oracle.conv2d(x, wt, L["bias"], stride=1)
        y2, s2 = oracle.conv2d(x, wt, L["bias"], stride=2)
        assert np.array_equal(y2, y1[:, :, ::2, ::2]) and np.array_equal(s2, s1[:, :, ::2, ::2])


def test_nhwc_is_transposed_nchw_and_points_equal_full():
    spec, L, x = tiny(5, 6, 7, 9, n=2, seed=17)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    y, s = oracle.conv2d(x, wt, L["bias"], relu=True)
    xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
    yh, sh = oracle.conv2d(xh, wt, L["bias"], relu=True, layout="nhwc")
    assert np.array_equal(yh.transpose(0, 3, 1, 2), y) and np.array_equal(sh.transpose(0, 3, 1, 2), s)
    pts = np.array([(n, f, oy, ox) for n in range(2) for f in range(6)
                    for oy in range(7) for ox in range(9)], np.int32)
    yp, sp = oracle.conv2d_points(x, wt, pts, L["bias"], relu=True)
    assert np.array_equal(yp.reshape(y.shape), y) and np.array_equal(sp.reshape(s.shape), s)
    yq, _ = oracle.conv2d_points(xh, wt, pts, L["bias"], relu=True, layout="nhwc")
    assert np.array_equal(yq, yp)
    # stride 2 points
    y2, _ = oracle.conv2d(x, wt, L["bias"], stride=2)
    pts2 = np.array([(1, 3, oy, ox) for oy in range(y2.shape[2]) for ox in range(y2.shape[3])], np.int32)
    assert np.array_equal(oracle.conv2d_points(x, wt, pts2, L["bias"], stride=2)[0].reshape(y2.shape[2:]),
                          y2[1, 3])


def test_tolerance_scale_properties():
    spec, L, x = tiny(5, 4, 6, 6, seed=23)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    y, s = oracle.conv2d(x, wt, L["bias"])
    assert np.all(s >= np.abs(y) - 1e-12)
    ya, _ = oracle.conv2d(np.abs(x), np.abs(wt), np.abs(L["bias"]))
    assert np.allclose(s, ya, rtol=1e-13)


def test_bf16_weight_rounding_matches_library_cast():
    rng = np.random.default_rng(8)
    w = rng.standard_normal((8, 8, 3, 3)).astype(np.float32)
    # exact ties and special values
    w.flat[0] = np.float32(1.00390625); w.flat[1] = np.float32(1.01171875)
    w.flat[2] = np.float32(-0.0); w.flat[3] = np.float32(3.0e-39); w.flat[4] = np.float32(65504.0)
    w.flat[5] = np.float32(3.3895313892515355e38)          # rounds up to +inf in bf16
    table = np.array([0x1FF], np.uint16)
    wt = oracle.masked_weights(w, np.zeros((8, 8), np.uint8), np.ones((8, 8), np.uint8), table, "bf16")
    ref = torch.from_numpy(w).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(wt, ref)
    assert oracle.bf16_bits(1.00390625) == 0x3F80 and oracle.bf16_bits(1.01171875) == 0x3F82


def test_maxpool_matches_library():
    rng = np.random.default_rng(1)
    for shape in [(2, 3, 8, 6), (1, 2, 7, 9)]:
        x = rng.standard_normal(shape).astype(np.float32)
        ref = torch.nn.functional.max_pool2d(torch.from_numpy(x), 2).numpy()
        assert np.array_equal(oracle.maxpool2x2(x), ref)
        xh = np.ascontiguousarray(x.transpose(0, 2, 3, 1))
        assert np.array_equal(oracle.maxpool2x2(xh, "nhwc").transpose(0, 3, 1, 2), ref)


def test_scp_table_matches_paper(golden_dir):
    """IDs 0-3 are the paper's four SCPs; their mean is [0 p 0; p 1 p; 0 p 0], p = 0.75."""
    import os
    mats, mean, cur, comp = {}, None, None, None
    for line in open(os.path.join(golden_dir, "scp_masks.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        tok = line.split()
        if tok[0] == "scp":
            cur = int(tok[1]); mats[cur] = []
        elif tok[0] == "mean":
            cur = "mean"; mean = []
        elif tok[0] == "pattern_compression":
            comp = float(tok[1])
        elif cur == "mean":
            mean.append([float(t) for t in tok])
        else:
            mats[cur].append([int(t) for t in tok])
    for i in range(4):
        m = sum(mats[i][r][s] << (3 * r + s) for r in range(3) for s in range(3))
        assert m == int(PATTERN_TABLE[i])
    avg = np.mean([np.array(mats[i], float) for i in range(4)], axis=0)
    assert np.array_equal(avg, np.array(mean))
    for m in PATTERN_TABLE:
        assert bin(int(m)).count("1") == 4 and (int(m) >> 4) & 1
    assert len(set(int(m) for m in PATTERN_TABLE)) == 12
    assert comp == 9 / 4
