"""GPU parity: pconv_conv2d (through the C ABI) against the CPU oracle, element by element.

Bar: packing and indices bit exact; fp32 outputs within 1e-4 * S, bf16 within 2e-2 * S, where
S = |bias| + sum |w||x| of that output.
"""
import numpy as np
import pytest

import oracle
import paper_1909_05073_amd as P
from pconv_inputs import LayerSpec, base_seed, config_layers, make_input, make_layer

from gpu_util import (assert_close, gather_points, gpu_conv, oracle_full, sample_points, say,
                      to_device)

pytestmark = pytest.mark.gpu

POLICIES = [1, 0]          # 1 = generic gather kernel, 0 = automatic (register-tiled / matrix-core where possible)
# (2 = register-tiled vector kernel required, 3 = matrix-core kernel required: bf16 handles only)


@pytest.fixture(autouse=True)
def _reset_policy():
    yield
    P.pconv_set_kernel_policy(0)
    P.pconv_debug_set_tiling(0, -1, -1)
    P.pconv_debug_set_spin_limit(0)


def check_full(spec, L, x, dtype, layout="nchw", stride=1, relu=False, use_bias=True, policy=0, what=""):
    say(f"[case] {what or spec.name} dtype={dtype} layout={layout} stride={stride} relu={relu} "
        f"policy={policy} x={x.shape}")
    P.pconv_set_kernel_policy(policy)
    y, h = gpu_conv(L, x, dtype, layout, stride, relu, use_bias)
    yr, sr = oracle_full(L, x, dtype, layout, stride, relu, use_bias)
    assert y.shape == yr.shape
    r = assert_close(y, yr, sr, dtype, what or spec.name)
    h.free()
    return r


@pytest.mark.parametrize("policy", POLICIES)
def test_config1_small_layer(policy):
    spec = config_layers(1)[0]
    L = make_layer(spec, base_seed(1)); x = make_input(spec, base_seed(1))
    check_full(spec, L, x, "f32", relu=False, policy=policy)
    check_full(spec, L, x, "f32", relu=True, use_bias=False, policy=policy)


@pytest.mark.parametrize("policy", POLICIES)
def test_config2_vgg_layer(policy):
    spec = config_layers(2)[0]
    L = make_layer(spec, base_seed(2)); x = make_input(spec, base_seed(2))
    check_full(spec, L, x, "f32", policy=policy)


def test_config3_vgg_stack_batch1_layerwise():
    """Every VGG-16 conv shape at batch 1 with fresh inputs, full output, ReLU fused."""
    for i, spec in enumerate(config_layers(3, batch=1)):
        L = make_layer(spec, base_seed(3) + 100 * i); x = make_input(spec, base_seed(3) + 100 * i)
        check_full(spec, L, x, "f32", relu=True)


def test_config3_vgg_chained_with_maxpool_batch2():
    """conv -> ReLU -> ... -> 2x2 max-pool chained on the device; each layer is checked against
    the oracle fed with the GPU's own previous activation, so tolerances do not compound."""
    import torch
    specs = config_layers(3, batch=2)
    x = make_input(specs[0], base_seed(3))
    cur = torch.from_numpy(x).cuda()
    for i, spec in enumerate(specs):
        L = make_layer(spec, base_seed(3) + 100 * i)
        say(f"[case] chained {spec.name} in={tuple(cur.shape)}")
        h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
        b = torch.from_numpy(L["bias"]).cuda()
        y = P.conv2d(h, cur, b, relu=True)
        torch.cuda.synchronize()
        xin = cur.cpu().numpy()
        wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
        rng = np.random.default_rng(i)
        pts = sample_points(rng, 2, spec.c_out, spec.h, spec.w, 3000)
        yr, sr = oracle.conv2d_points(xin, wt, pts, L["bias"], relu=True)
        assert_close(gather_points(y.cpu().numpy().astype(np.float64), pts, "nchw"), yr, sr, "f32", spec.name)
        h.free()
        if spec.pool_after:
            p = P.maxpool2x2(y)
            torch.cuda.synchronize()
            assert np.array_equal(p.cpu().numpy(), oracle.maxpool2x2(y.cpu().numpy()))
            cur = p
        else:
            cur = y
    assert tuple(cur.shape) == (2, 512, 7, 7)


@pytest.mark.parametrize("idx", [0, 2, 4, 7, 10, 1, 5, 9, 12])
def test_config3_vgg_batch32_sampled(idx):
    """Bench launch configuration (batch 32) on sampled outputs the oracle computes one by one:
    every layer shape that the benchmark runs through pconv_conv2d."""
    spec = config_layers(3, batch=32)[idx]
    L = make_layer(spec, base_seed(3) + 100 * idx); x = make_input(spec, base_seed(3) + 100 * idx)
    say(f"[case] {spec.name} N=32 sampled")
    y, h = gpu_conv(L, x, "f32", relu=True)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    pts = sample_points(np.random.default_rng(idx), 32, spec.c_out, spec.h, spec.w, 20000)
    yr, sr = oracle.conv2d_points(x, wt, pts, L["bias"], relu=True)
    assert_close(gather_points(y, pts, "nchw"), yr, sr, "f32", spec.name)
    h.free()


@pytest.mark.parametrize("idx", [1, 3, 6, 9])
def test_config3_vgg_batch32_fused_pool_sampled(idx):
    """The fused convolution + max-pool launches of the benchmark (batch 32) on sampled pooled
    outputs: the oracle computes the four convolution outputs under each of them one by one."""
    import torch
    spec = config_layers(3, batch=32)[idx]
    assert spec.pool_after
    L = make_layer(spec, base_seed(3) + 100 * idx); x = make_input(spec, base_seed(3) + 100 * idx)
    say(f"[case] {spec.name}+pool N=32 sampled")
    h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    y = P.conv2d_pool2x2(h, to_device(x, "f32"), torch.from_numpy(L["bias"]).cuda(), relu=True)
    torch.cuda.synchronize()
    y = y.cpu().numpy().astype(np.float64)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    pp = sample_points(np.random.default_rng(100 + idx), 32, spec.c_out, spec.h // 2, spec.w // 2, 5000)
    ref = np.full(len(pp), -np.inf); s_ref = np.zeros(len(pp))
    for dy in (0, 1):
        for dx in (0, 1):
            pts = pp.copy(); pts[:, 2] = 2 * pp[:, 2] + dy; pts[:, 3] = 2 * pp[:, 3] + dx
            yr, sr = oracle.conv2d_points(x, wt, pts.astype(np.int32), L["bias"], relu=True)
            ref = np.maximum(ref, yr); s_ref = np.maximum(s_ref, sr)
    assert_close(gather_points(y, pp, "nchw"), ref, s_ref, "f32", spec.name + "+pool")
    h.free()


@pytest.mark.parametrize("w", [32760, 32776])
def test_input_just_below_and_above_2_gib(w):
    """The fp32 NCHW kernel stages with range-checked buffer loads, which address at most 2^31 - 1
    bytes; a larger input takes the register-staging kernel.  One layer on either side of the
    limit (2 x 8192 x w floats), on sampled outputs: byte offsets close to 2^31 in the first case,
    the change of kernels in the second."""
    import torch
    n, c_in, c_out, h = 1, 2, 4, 8192
    nbytes = n * c_in * h * w * 4
    assert (nbytes < 2**31) == (w == 32760)
    spec = LayerSpec("limit", n, c_in, c_out, h, w, pattern_dist="uniform", count_dist="all")
    L = make_layer(spec, 4242)
    say(f"[case] input of {nbytes} bytes (limit {2**31}), w={w}")
    rng = np.random.default_rng(77)
    x = rng.standard_normal((n, c_in, h, w), dtype=np.float32)
    hd = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    y = P.conv2d(hd, torch.from_numpy(x).cuda(), torch.from_numpy(L["bias"]).cuda(), relu=False)
    torch.cuda.synchronize()
    pts = sample_points(rng, n, c_out, h, w, 20000)
    # the last rows and columns as well: the highest addresses of the tensor
    tail = np.array([(0, f, yy, xx) for f in range(c_out) for yy in (h - 2, h - 1) for xx in range(w - 6, w)], np.int32)
    pts = np.concatenate([pts, tail])
    idx = torch.from_numpy(pts.astype(np.int64)).cuda()
    got = y[idx[:, 0], idx[:, 1], idx[:, 2], idx[:, 3]].cpu().numpy().astype(np.float64)
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    yr, sr = oracle.conv2d_points(x, wt, pts, L["bias"], relu=False)
    assert_close(got, yr, sr, "f32", f"input of {nbytes} bytes")
    hd.free()


@pytest.mark.parametrize("policy", [0, 2])
def test_config4_resnet_bf16(policy):
    """All sixteen ResNet-50 3x3 layers (stride 2 included), bf16 in/out, fp32 accumulate: as the
    library chooses (the matrix-core kernel at this density) and on the vector kernel."""
    seen = set()
    P.pconv_set_kernel_policy(policy)
    shares = []
    for i, spec in enumerate(config_layers(4, batch=32)):
        key = (spec.c_in, spec.h, spec.stride)
        L = make_layer(spec, base_seed(4) + i); x = make_input(spec, base_seed(4) + i)
        say(f"[case] {spec.name} N=32 bf16 sampled")
        y, h = gpu_conv(L, x, "bf16", stride=spec.stride, relu=True)
        wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"], "bf16")
        pts = sample_points(np.random.default_rng(i), 32, spec.c_out, spec.h_out, spec.w_out, 8000)
        yr, sr = oracle.conv2d_points(x, wt, pts, L["bias"], stride=spec.stride, relu=True)
        yg = gather_points(y, pts, "nchw")
        assert_close(yg, yr, sr, "bf16", spec.name)
        # secondary figure: share of the sampled outputs within 2e-2 of the oracle value itself
        big = np.abs(yr) > 0
        shares.append(float(np.mean(np.abs(yg - yr)[big] <= 2e-2 * np.abs(yr[big]))))
        if key not in seen:                      # full-output check at batch 2 once per shape
            seen.add(key)
            check_full(spec, L, x[:2], "bf16", stride=spec.stride, relu=True, policy=policy, what=spec.name + "_n2")
        h.free()
    say(f"[info] config 4, policy {policy}: share of non-zero sampled outputs with |err| <= 2e-2*|y|: "
        f"min {min(shares):.4f} mean {np.mean(shares):.4f} over {len(shares)} layers")


def test_config5_stress_imbalanced():
    spec = config_layers(5)[0]
    L = make_layer(spec, base_seed(5)); x = make_input(spec, base_seed(5))
    say("[case] config5 N=64 sampled")
    y, h = gpu_conv(L, x, "f32")
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    pts = sample_points(np.random.default_rng(5), 64, 512, 28, 28, 30000)
    # every filter's first pixel too: heavy and near-empty filters alike
    allf = np.array([(63, f, 27, 27) for f in range(512)], np.int32)
    pts = np.concatenate([pts, allf])
    yr, sr = oracle.conv2d_points(x, wt, pts, L["bias"])
    assert_close(gather_points(y, pts, "nchw"), yr, sr, "f32", spec.name)
    check_full(spec, L, x[:2], "f32", what="config5_n2")
    check_full(spec, L, x[:1], "f32", policy=1, what="config5_n1_generic")
    h.free()


EDGE_SHAPES = [  # (n, c_in, c_out, h, w)
    (1, 1, 1, 1, 1), (2, 3, 5, 5, 3), (1, 8, 8, 13, 13), (3, 5, 17, 7, 9), (1, 16, 9, 4, 33),
    (2, 7, 64, 14, 14), (1, 9, 70, 30, 18), (1, 4, 8, 3, 70),
]


@pytest.mark.parametrize("policy", POLICIES + [2, 3])   # 2 = register-tiled kernel for every call (small stride-2 layers too)
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
@pytest.mark.parametrize("stride", [1, 2])
def test_ragged_shapes_layouts_strides(policy, dtype, layout, stride):
    if policy == 3 and dtype == "f32":
        pytest.skip("the matrix-core kernel serves bf16 only (see test_matrix_core_kernel_rejects_fp32)")
    for j, (n, ci, co, h, w) in enumerate(EDGE_SHAPES):
        spec = LayerSpec(f"edge{j}", n, ci, co, h, w, stride=stride, dtype=dtype, num_patterns=12,
                         pattern_dist="uniform", keep_div=2.0, count_dist="bernoulli")
        L = make_layer(spec, 1000 + j); x = make_input(spec, 1000 + j, layout)
        check_full(spec, L, x, dtype, layout, stride, relu=bool(j & 1), use_bias=bool(j & 2), policy=policy)


@pytest.mark.parametrize("waves,ks_log2", [(0, -1), (8, 0), (16, 1), (16, 2)])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_stride2_through_the_tiled_kernel(waves, ks_log2, dtype):
    """Stride 2 on the register-tiled kernel (full-resolution sums, every other output stored) in
    every workgroup shape, odd and even sizes, several chunks and filter groups."""
    for j, (n, ci, co, h, w) in enumerate([(2, 37, 150, 14, 14), (1, 64, 64, 29, 31), (3, 19, 70, 9, 22), (1, 130, 33, 7, 7)]):
        spec = LayerSpec(f"s2_{j}", n, ci, co, h, w, stride=2, dtype=dtype)
        L = make_layer(spec, 3000 + j); x = make_input(spec, 3000 + j)
        P.pconv_debug_set_tiling(waves, ks_log2, -1)
        check_full(spec, L, x, dtype, "nchw", 2, relu=bool(j & 1), policy=2, what=f"{spec.name} waves={waves} ks={ks_log2}")


TILING_SHAPES = [  # (n, c_in, c_out, h, w): several chunks and filter groups, ragged in every dimension
    (2, 37, 150, 14, 14), (1, 64, 64, 28, 28), (3, 19, 70, 9, 21), (1, 130, 33, 7, 7), (2, 8, 8, 4, 4),
]


@pytest.mark.parametrize("split_units", [0, 1, 2])
@pytest.mark.parametrize("ks_log2", [0, 1, 2])
@pytest.mark.parametrize("waves", [8, 16])
def test_tiled_kernel_every_workgroup_shape_and_channel_split(waves, ks_log2, split_units):
    """The register-tiled kernel in both workgroup shapes, all three channel splits inside a
    workgroup, with and without units shared between workgroups: choices the automatic
    selection only makes for particular layer sizes."""
    P.pconv_debug_set_tiling(waves, ks_log2, split_units)
    for j, (n, ci, co, h, w) in enumerate(TILING_SHAPES):
        for dtype, layout in (("f32", "nchw"), ("bf16", "nhwc")):
            spec = LayerSpec(f"tiling{j}", n, ci, co, h, w, dtype=dtype, num_patterns=12,
                             pattern_dist="uniform", keep_div=2.0, count_dist="bernoulli")
            L = make_layer(spec, 2000 + j); x = make_input(spec, 2000 + j, layout)
            check_full(spec, L, x, dtype, layout, 1, relu=bool(j & 1), policy=2,
                       what=f"tiling{j}_w{waves}_ks{ks_log2}_split{split_units}")


# Layers whose pieces walk more than 64 chunks of input channels (the bounds of the chunks sit one
# per lane and are re-read every 64 chunks): c_in above 512 with 8-channel chunks, above 256 with
# the 8-wave shape's 4-channel chunks.  Small images keep the oracle cheap.
@pytest.mark.parametrize("waves,c_in,split_units", [(16, 520, 0), (16, 520, 1), (16, 1030, 0), (16, 1030, 1),
                                                     (8, 300, 0), (8, 300, 1)])
def test_more_than_64_chunks_of_input_channels(waves, c_in, split_units):
    P.pconv_debug_set_tiling(waves, 0, split_units)
    for j, (n, co, h, w) in enumerate([(1, 24, 8, 8), (2, 70, 5, 12)]):
        spec = LayerSpec(f"deep{j}", n, c_in, co, h, w, num_patterns=8, pattern_dist="uniform",
                         keep_div=3.0, count_dist="bernoulli")
        L = make_layer(spec, 4000 + j); x = make_input(spec, 4000 + j)
        check_full(spec, L, x, "f32", "nchw", 1, relu=bool(j), policy=2,
                   what=f"deep{j}_cin{c_in}_w{waves}_split{split_units}")


# Units shared between workgroups on layers of several tiles, also where the image width is no
# multiple of 4: there the last patch of a row overlaps its neighbour, and when the two lie in
# different tiles the library must not let their workgroups pass partial sums through the
# columns they share (it then keeps whole units).
@pytest.mark.parametrize("split_units", [-1, 1, 2])
@pytest.mark.parametrize("shape", [(4, 256, 64, 18, 18), (32, 256, 256, 10, 10), (3, 96, 64, 20, 24),
                                   (6, 72, 128, 14, 14), (2, 64, 64, 30, 26)])
def test_shared_units_on_several_tiles(shape, split_units):
    n, ci, co, h, w = shape
    P.pconv_debug_set_tiling(0, -1, split_units)
    spec = LayerSpec("multitile", n, ci, co, h, w)
    L = make_layer(spec, 5000 + h); x = make_input(spec, 5000 + h)
    check_full(spec, L, x, "f32", "nchw", 1, relu=True, policy=2, what=f"multitile{shape}_split{split_units}")


def test_four_scp_table():
    """A table of the paper's four Sparse Convolution Patterns alone (the 4-pattern row of the
    pattern-count experiment)."""
    for j, (n, ci, co, h, w) in enumerate([(2, 40, 70, 14, 14), (1, 64, 64, 28, 28)]):
        spec = LayerSpec(f"scp4_{j}", n, ci, co, h, w, num_patterns=4, pattern_dist="uniform")
        L = make_layer(spec, 6000 + j); x = make_input(spec, 6000 + j)
        assert len(L["table"]) == 4
        for policy in POLICIES:
            check_full(spec, L, x, "f32", relu=True, policy=policy, what=f"scp4_{j}")


def test_tables_of_random_masks():
    """Pattern tables drawn at random, as in the paper's pattern-count experiment ("random patterns
    with 4 non-zero elements"): 4-tap masks with the centre (one work item per kernel), 4-tap masks
    without it, and masks of 2 to 7 taps (split into several items at pack time)."""
    rng = np.random.default_rng(99)
    centred = [m for m in range(512) if bin(m).count("1") == 4 and (m >> 4) & 1]
    free4 = [m for m in range(512) if bin(m).count("1") == 4 and not (m >> 4) & 1]
    other = [m for m in range(1, 512) if bin(m).count("1") in (2, 3, 5, 6, 7)]
    tables = [rng.choice(centred, 8, replace=False), rng.choice(centred, 16, replace=False),
              rng.choice(free4, 8, replace=False), rng.choice(other, 12, replace=False)]
    for j, table in enumerate(tables):
        table = np.asarray(table, np.uint16)
        f, c = 72, 40
        L = dict(w=rng.standard_normal((f, c, 3, 3)).astype(np.float32),
                 bias=rng.standard_normal(f).astype(np.float32),
                 pattern_id=rng.integers(0, len(table), (f, c)).astype(np.uint8),
                 conn=(rng.random((f, c)) < 0.4).astype(np.uint8), table=table)
        spec = LayerSpec(f"randtable{j}", 2, c, f, 13, 16)
        x = make_input(spec, 8000 + j) - 0.3
        for policy in POLICIES:
            check_full(spec, L, x, "f32", relu=bool(j & 1), policy=policy, what=f"random table {j}")
        h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], table, "f32")
        _, records = P.pconv_debug_export_blocks(h)
        kept = int(L["conn"].sum())
        say(f"[info] random table {j}: {int(records.sum())} work items for {kept} kernels")
        if j < 2:
            assert int(records.sum()) == kept         # one item per kernel for centred 4-tap masks
        h.free()


def test_expired_wait_is_reported_by_the_next_call():
    """Error path, forced from the host: with a spin limit of 1 every bounded wait inside the tiled
    kernel gives up at once.  The kernels still run to their end; the handle reports the failure
    on the next call (which launches nothing) and works again afterwards."""
    import torch
    spec = config_layers(2)[0]                       # shared units: both kinds of wait are used
    L = make_layer(spec, base_seed(2)); x = make_input(spec, base_seed(2))
    h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    xd = to_device(x, "f32"); b = torch.from_numpy(L["bias"]).cuda()
    good = P.conv2d(h, xd, b, relu=True).clone()
    torch.cuda.synchronize()
    P.pconv_get_async_error(h)                       # nothing to report
    say("[case] spin limit 1")
    P.pconv_debug_set_spin_limit(1)
    P.conv2d(h, xd, b, relu=True)
    torch.cuda.synchronize()
    P.pconv_debug_set_spin_limit(0)
    with pytest.raises(P.PconvError) as e:
        P.conv2d(h, xd, b, relu=True)
    assert e.value.status == P.HIP_ERROR and "bounded wait" in str(e.value)
    P.pconv_get_async_error(h)                       # reported once
    y = P.conv2d(h, xd, b, relu=True)
    torch.cuda.synchronize()
    assert torch.equal(y, good)
    P.pconv_get_async_error(h)
    h.free()


@pytest.mark.parametrize("policy", POLICIES)
def test_degenerate_filters_and_mixed_masks(policy):
    rng = np.random.default_rng(7)
    f, c = 20, 12
    table = np.array([0x1FF, 0x010, 0x03A, 0x145, 0x0B2, 0x001, 0x100], np.uint16)
    L = dict(w=rng.standard_normal((f, c, 3, 3)).astype(np.float32),
             bias=rng.standard_normal(f).astype(np.float32),
             pattern_id=rng.integers(0, len(table), (f, c)).astype(np.uint8),
             conn=rng.integers(0, 2, (f, c)).astype(np.uint8), table=table)
    L["conn"][3] = 0; L["conn"][11] = 0      # filters with no kernel: output = act(bias)
    L["conn"][5] = 1                          # filter with every kernel
    spec = LayerSpec("mixed", 2, c, f, 9, 10)
    x = make_input(spec, 5) - 0.4
    check_full(spec, L, x, "f32", relu=False, policy=policy, what="mixed masks")
    check_full(spec, L, x, "f32", relu=True, stride=2, policy=policy, what="mixed masks s2")
    L["conn"][:] = 0                          # nothing kept at all
    check_full(spec, L, x, "f32", relu=False, policy=policy, what="empty layer")


POOL_SHAPES = [  # (n, c_in, c_out, h, w): even widths; odd and tiny heights; several tiles and filter groups
    (2, 16, 70, 14, 14), (1, 37, 64, 28, 28), (3, 8, 9, 7, 6), (1, 5, 130, 2, 4), (2, 24, 16, 9, 34), (1, 3, 64, 32, 32),
]


@pytest.mark.parametrize("waves,ks_log2", [(0, -1), (8, 0), (16, 1), (16, 2)])
def test_fused_maxpool_equals_conv_then_pool(waves, ks_log2):
    """pconv_conv2d_pool2x2 against the oracle's convolution followed by its max-pool; a pooled
    value may be off by what the largest of its four inputs may be off."""
    import torch
    # (units are not shared between workgroups here, which the fused call never does either: then
    # the two ways add in the same order and must agree bit for bit)
    P.pconv_debug_set_tiling(waves, ks_log2, 0)
    for j, (n, ci, co, h, w) in enumerate(POOL_SHAPES):
        spec = LayerSpec(f"pool{j}", n, ci, co, h, w, num_patterns=12, pattern_dist="uniform",
                         keep_div=2.0, count_dist="bernoulli")
        L = make_layer(spec, 3000 + j); x = make_input(spec, 3000 + j)
        for relu in (False, True):
            say(f"[case] pool{j} waves={waves} ks={ks_log2} relu={relu} x={x.shape}")
            hd = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
            b = torch.from_numpy(L["bias"]).cuda()
            y = P.conv2d_pool2x2(hd, to_device(x, "f32"), b, relu=relu)
            torch.cuda.synchronize()
            yr, sr = oracle_full(L, x, "f32", "nchw", 1, relu, True)
            pr = oracle.maxpool2x2(yr.astype(np.float32)).astype(np.float64)
            # reference pooled in fp64 to keep the comparison exact
            hh, ww = h // 2, w // 2
            pr = yr[:, :, :2 * hh, :2 * ww].reshape(n, co, hh, 2, ww, 2).max(axis=(3, 5))
            ps = sr[:, :, :2 * hh, :2 * ww].reshape(n, co, hh, 2, ww, 2).max(axis=(3, 5))
            assert tuple(y.shape) == pr.shape
            assert_close(y.cpu().numpy().astype(np.float64), pr, ps, "f32", f"pool{j}")
            # and bit for bit what the two separate calls give
            y2 = P.maxpool2x2(P.conv2d(hd, to_device(x, "f32"), b, relu=relu))
            torch.cuda.synchronize()
            assert torch.equal(y, y2), f"pool{j}: fused and separate results differ"
            hd.free()


MFMA_SHAPES = [  # (n, c_in, c_out, h, w, stride): several channel blocks, ragged filter blocks, tiles of every kind
    (2, 64, 64, 56, 56, 1), (3, 40, 70, 28, 28, 1), (5, 96, 33, 14, 14, 1), (9, 130, 64, 7, 7, 1),
    (2, 64, 96, 56, 56, 2), (3, 48, 40, 29, 31, 2), (1, 16, 8, 3, 300, 1), (1, 8, 160, 40, 9, 1),
]


@pytest.mark.parametrize("layout", ["nchw", "nhwc"])
def test_matrix_core_kernel_shapes(layout):
    """The bf16 matrix-core kernel on every kind of tile it builds (rows of one image, whole images,
    several images, split rows), both strides, channel and filter counts off the block sizes."""
    for j, (n, ci, co, h, w, stride) in enumerate(MFMA_SHAPES):
        spec = LayerSpec(f"mfma{j}", n, ci, co, h, w, stride=stride, dtype="bf16", keep_div=2.5)
        L = make_layer(spec, 7000 + j); x = make_input(spec, 7000 + j, layout)
        check_full(spec, L, x, "bf16", layout, stride, relu=bool(j & 1), use_bias=not (j & 2), policy=3,
                   what=f"mfma{j}_{layout}")


def test_matrix_core_kernel_skips_empty_weight_blocks():
    """Connectivity so sparse that whole (tap, 16 channels, 32 filters) blocks hold no weight: the
    kernel skips them; and a layer with nothing kept at all."""
    rng = np.random.default_rng(11)
    f, c = 70, 100
    spec = LayerSpec("mfma_sparse", 2, c, f, 12, 12, dtype="bf16", num_patterns=4, pattern_dist="uniform")
    L = make_layer(spec, 7100)
    L["conn"][:] = 0
    L["conn"][rng.integers(0, f, 40), rng.integers(0, c, 40)] = 1
    L["conn"][:, 32:64] = 0                          # a whole block of channels unused
    x = make_input(spec, 7100)
    check_full(spec, L, x, "bf16", relu=False, policy=3, what="mfma sparse")
    L["conn"][:] = 0
    check_full(spec, L, x, "bf16", relu=True, policy=3, what="mfma empty")


def test_matrix_core_kernel_rejects_fp32():
    import torch
    spec = config_layers(1)[0]
    L = make_layer(spec, base_seed(1))
    h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    x = torch.zeros(1, 16, 16, 16, device="cuda"); y = torch.zeros_like(x)
    P.pconv_set_kernel_policy(3)
    with pytest.raises(P.PconvError) as e:
        P.pconv_conv2d(h, x.data_ptr(), y.data_ptr(), 0, 1, 16, 16)
    assert e.value.status == P.UNSUPPORTED
    h.free()


def test_fused_maxpool_rejects_what_it_cannot_do():
    import torch
    spec = LayerSpec("poolerr", 1, 4, 8, 6, 7, num_patterns=12)
    L = make_layer(spec, 7)
    hd = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    x = torch.zeros((1, 4, 6, 7), device="cuda"); y = torch.zeros((1, 8, 3, 3), device="cuda")
    with pytest.raises(P.PconvError) as e:
        P.pconv_conv2d_pool2x2(hd, x.data_ptr(), y.data_ptr(), 0, 1, 6, 7)         # odd width
    assert e.value.status == P.UNSUPPORTED
    x = torch.zeros((1, 6, 8, 4), device="cuda")
    with pytest.raises(P.PconvError) as e:
        P.pconv_conv2d_pool2x2(hd, x.data_ptr(), y.data_ptr(), 0, 1, 6, 8, P.NHWC)  # NHWC
    assert e.value.status == P.UNSUPPORTED
    P.pconv_set_kernel_policy(1)
    x = torch.zeros((1, 4, 6, 8), device="cuda")
    with pytest.raises(P.PconvError) as e:
        P.pconv_conv2d_pool2x2(hd, x.data_ptr(), y.data_ptr(), 0, 1, 6, 8)         # generic kernel forced
    assert e.value.status == P.UNSUPPORTED
    with pytest.raises(P.PconvError) as e:
        P.pconv_conv2d_pool2x2(hd, 0, y.data_ptr(), 0, 1, 6, 8)
    assert e.value.status == P.INVALID_ARG
    hd.free()


def test_dense_mask_equals_library_conv():
    """All-ones mask + full connectivity on the GPU against a library dense convolution."""
    import torch
    rng = np.random.default_rng(2)
    w = rng.standard_normal((16, 6, 3, 3)).astype(np.float32)
    x = rng.standard_normal((2, 6, 12, 20)).astype(np.float32)
    L = dict(w=w, bias=np.zeros(16, np.float32), pattern_id=np.zeros((16, 6), np.uint8),
             conn=np.ones((16, 6), np.uint8), table=np.array([0x1FF], np.uint16))
    y, h = gpu_conv(L, x, "f32", use_bias=False)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), padding=1)
    s = torch.nn.functional.conv2d(torch.from_numpy(x).double().abs(), torch.from_numpy(w).double().abs(),
                                   padding=1)
    assert_close(y, ref.numpy(), s.numpy(), "f32", "dense")
    h.free()


def test_device_pack_bit_exact_and_unpack_roundtrip():
    for cfg, dtype in [(2, "f32"), (5, "f32"), (4, "bf16")]:
        spec = config_layers(cfg)[0]
        L = make_layer(spec, base_seed(cfg))
        say(f"[case] pack cfg{cfg} {dtype}")
        h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], dtype)
        got = P.pconv_debug_export(h)
        ref = oracle.pack(L["w"], L["pattern_id"], L["conn"], L["table"], dtype)
        for k in ("perm", "row_ptr", "pat_cnt", "cin", "vals"):
            assert got[k].tobytes() == ref[k].tobytes(), k
        wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"], dtype).astype(np.float32)
        assert np.array_equal(P.pconv_debug_unpack(h).view(np.uint32), wt.view(np.uint32))
        info = h.info()
        assert info.device_bytes > 0 and info.nnz == len(ref["vals"])
        h.free()


def test_run_to_run_bit_identical_and_stream():
    import torch
    spec = config_layers(2)[0]
    L = make_layer(spec, base_seed(2)); x = make_input(spec, base_seed(2))
    h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    xd = to_device(x, "f32"); b = torch.from_numpy(L["bias"]).cuda()
    y0 = P.conv2d(h, xd, b).clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        y1 = P.conv2d(h, xd, b)
    side.synchronize()
    y2 = P.conv2d(h, xd, b)
    torch.cuda.synchronize()
    assert torch.equal(y0, y1) and torch.equal(y0, y2)
    h.free()


def test_concurrent_calls_on_one_handle_with_shared_units():
    """Two streams run the same handle at the same time on a layer whose workgroups share units
    (they signal each other through per-call words of the handle): every result must equal, bit
    for bit, what the same call gives alone."""
    import torch
    spec = config_layers(2)[0]                       # 256 -> 256 at 56x56, batch 1: 16 units, shared
    L = make_layer(spec, base_seed(2))
    h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    b = torch.from_numpy(L["bias"]).cuda()
    xs = [to_device(make_input(spec, base_seed(2) + 7 * k), "f32") for k in range(2)]
    refs = [P.conv2d(h, x, b, relu=True).clone() for x in xs]
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [[], []]
    for s in streams:
        s.wait_stream(torch.cuda.current_stream())
    say("[case] 2 streams x 12 overlapping calls on one handle")
    for it in range(12):
        for k in range(2):
            with torch.cuda.stream(streams[k]):
                outs[k].append(P.conv2d(h, xs[k], b, relu=True))
    for s in streams:
        s.synchronize()
    for k in range(2):
        for it, y in enumerate(outs[k]):
            assert torch.equal(y, refs[k]), f"stream {k}, call {it}: differs from the call run alone"
    h.free()


def test_gpu_argument_errors():
    import torch
    spec = config_layers(1)[0]
    L = make_layer(spec, base_seed(1))
    h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    x = torch.zeros(1, 16, 16, 16, device="cuda"); y = torch.zeros_like(x)
    with pytest.raises(P.PconvError) as e:
        P.pconv_conv2d(h, x.data_ptr(), y.data_ptr(), 0, 1, 16, 16, act_dtype=P.BF16)
    assert e.value.status == P.INVALID_ARG
    with pytest.raises(P.PconvError):
        P.pconv_conv2d(h, x.data_ptr(), y.data_ptr(), 0, 1, 16, 16, stride=4)
    with pytest.raises(P.PconvError):
        P.pconv_conv2d(h, x.data_ptr(), y.data_ptr(), 0, 1 << 20, 1 << 10, 1 << 10)
    P.pconv_conv2d(h, x.data_ptr(), y.data_ptr(), 0, 1, 16, 16)     # still usable afterwards
    torch.cuda.synchronize()
    h.free()
