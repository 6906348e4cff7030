"""pconv_conv2d_static (the entry point for callers that cannot let the library allocate: its
hand-over words live in a static device array of the code object) against pconv_conv2d, through
the C ABI: same kernels, same order of additions, so the outputs must agree bit for bit - and
with the oracle within the fp32 bar.  Two calls in a row, the second on a smaller input."""
import numpy as np
import pytest

import oracle
import paper_1909_05073_amd as P
from pconv_inputs import LayerSpec, base_seed, config_layers, make_input, make_layer

from gpu_util import assert_close, say, to_device

pytestmark = pytest.mark.gpu


def test_static_scratch_entry_point_two_calls_second_smaller():
    import torch
    spec = config_layers(2)[0]                       # 256 -> 256 at 56x56, batch 1: workgroups share units
    L = make_layer(spec, base_seed(2))
    h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32")
    b = torch.from_numpy(L["bias"]).cuda()
    wt = oracle.masked_weights(L["w"], L["pattern_id"], L["conn"], L["table"])
    stream = torch.cuda.current_stream().cuda_stream
    for k, (hh, ww) in enumerate([(56, 56), (28, 20)]):
        x = make_input(LayerSpec("s", 1, 256, 256, hh, ww), base_seed(2) + k)
        xd = to_device(x, "f32")
        say(f"[case] pconv_conv2d_static call {k}: x={x.shape}")
        ref = P.conv2d(h, xd, b, relu=True)
        y = torch.full_like(ref, float("nan"))
        P.pconv_conv2d_static(h, xd.data_ptr(), y.data_ptr(), b.data_ptr(), 1, hh, ww, 1, 1, P.NCHW, P.F32,
                              True, stream)
        torch.cuda.synchronize()
        assert torch.equal(y, ref), f"call {k}: static-scratch result differs from pconv_conv2d"
        yr, sr = oracle.conv2d(x, wt, L["bias"], relu=True)
        assert_close(y.cpu().numpy().astype(np.float64), yr, sr, "f32", f"static call {k}")
    P.pconv_get_async_error(h)
    h.free()
