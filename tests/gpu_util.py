"""Helpers of the GPU parity tests: run one layer through the C ABI, compare with the oracle."""
import sys

import numpy as np

import oracle
import paper_1909_05073_amd as P

TOL = {"f32": 1e-4, "bf16": 2e-2}     # |y_gpu - y_oracle| <= TOL * S,  S = |b| + sum |w||x|


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def to_device(x_np, dtype):
    import torch
    t = torch.from_numpy(x_np).cuda()
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def gpu_conv(L, x_np, dtype="f32", layout="nchw", stride=1, relu=False, use_bias=True, handle=None):
    """Returns (y as float64 numpy in the layout of x, handle)."""
    import torch
    h = handle or P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], dtype)
    x = to_device(x_np, dtype)
    b = torch.from_numpy(L["bias"]).cuda() if use_bias else None
    y = P.conv2d(h, x, b, stride=stride, relu=relu, layout=layout)
    torch.cuda.synchronize()
    return y.float().cpu().numpy().astype(np.float64), h


def oracle_full(L, x_np, dtype="f32", layout="nchw", stride=1, relu=False, use_bias=True):
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"], dtype)
    return oracle.conv2d(x_np, wt, L["bias"] if use_bias else None, stride=stride, pad=1, relu=relu,
                         layout=layout)


def assert_close(y_gpu, y_ref, s_ref, dtype, what):
    err = np.abs(y_gpu - y_ref)
    bound = TOL[dtype] * s_ref
    ratio = float(np.max(err / np.maximum(s_ref, 1e-30))) if err.size else 0.0
    bad = np.argwhere(err > bound + 1e-30)
    assert bad.size == 0, (f"{what}: {len(bad)} of {err.size} outputs outside {TOL[dtype]}*S; worst "
                           f"err/S = {ratio:.3e} at {tuple(bad[0])}: gpu {y_gpu[tuple(bad[0])]} "
                           f"ref {y_ref[tuple(bad[0])]}")
    return ratio


def sample_points(rng, n, f, ho, wo, count):
    """Random output points plus all four corners / border midpoints of a few (n, f) planes."""
    pts = np.stack([rng.integers(0, n, count), rng.integers(0, f, count),
                    rng.integers(0, ho, count), rng.integers(0, wo, count)], axis=1)
    edge = []
    for nn in {0, n - 1}:
        for ff in {0, f // 2, f - 1}:
            for yy in {0, ho // 2, ho - 1}:
                for xx in {0, wo // 2, wo - 1}:
                    edge.append((nn, ff, yy, xx))
    return np.concatenate([pts, np.array(edge)], axis=0).astype(np.int32)


def gather_points(y, pts, layout):
    if layout == "nchw":
        return y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
    return y[pts[:, 0], pts[:, 2], pts[:, 3], pts[:, 1]]
