"""Host logic of pconv_pack against the oracle's reference packer (no GPU needed)."""
import ctypes as C
import re
import os

import numpy as np
import pytest

import oracle
import paper_1909_05073_amd as P
from pconv_inputs import LayerSpec, base_seed, config_layers, make_layer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "pconv.h")).read()
    declared = set(re.findall(r"\b(pconv_[a-z0-9_]+)\s*\(", text))
    declared -= {"pconv_handle"}
    assert declared == set(P.EXPORTED_SYMBOLS)
    L = P.lib()
    for name in declared:
        assert getattr(L, name) is not None


def _layers():
    out = []
    for cfg in (1, 2, 5):
        spec = config_layers(cfg)[0]
        out.append((f"cfg{cfg}", make_layer(spec, base_seed(cfg))))
    spec = config_layers(3)[0]                           # dense 3->64 first VGG layer
    out.append(("vgg_conv1", make_layer(spec, base_seed(3))))
    spec = config_layers(4)[4]
    out.append(("rn50_128", make_layer(spec, base_seed(4) + 4)))
    rng = np.random.default_rng(0)                       # mixed popcounts + degenerate filters
    f, c = 9, 11
    L = dict(w=rng.standard_normal((f, c, 3, 3)).astype(np.float32),
             pattern_id=rng.integers(0, 4, (f, c)).astype(np.uint8),
             conn=rng.integers(0, 2, (f, c)).astype(np.uint8),
             table=np.array([0x1FF, 0x010, 0x03A, 0x145], np.uint16))
    L["conn"][3] = 0; L["conn"][5] = 1
    L["pattern_id"][3] = 200                              # don't-care on removed kernels
    out.append(("mixed", L))
    return out


@pytest.mark.parametrize("wdtype", ["f32", "bf16"])
@pytest.mark.parametrize("name,L", _layers(), ids=[n for n, _ in _layers()])
def test_pack_matches_reference_packer_bit_exactly(name, L, wdtype):
    w = L["w"].copy()
    kf, kc = np.nonzero(L["conn"])
    w[kf[0], kc[0]] = np.array([-0.0, 1e-41, 1.00390625, 1.01171875, -1e-39, 3.0, 65504.0, -2.5, 0.0],
                               np.float32).reshape(3, 3)
    h = P.pconv_pack(w, L["pattern_id"], L["conn"], L["table"], wdtype, host_only=True)
    got = P.pconv_debug_export(h)
    ref = oracle.pack(w, L["pattern_id"], L["conn"], L["table"], wdtype)
    for k in ("perm", "row_ptr", "pat_cnt", "cin", "vals"):
        assert got[k].dtype == ref[k].dtype and got[k].tobytes() == ref[k].tobytes(), k
    info = h.info()
    assert info.kept_kernels == int((L["conn"] != 0).sum()) == len(ref["cin"])
    assert info.nnz == len(ref["vals"])
    # the exported layout unpacks (by the oracle's inverse) to the masked weights exactly
    back = oracle.unpack(got, L["table"], w.shape[1], wdtype)
    wt = oracle.masked_weights(w, L["pattern_id"], L["conn"], L["table"], wdtype).astype(np.float32)
    assert np.array_equal(back.view(np.uint32), wt.view(np.uint32))
    h.free()


def test_pack_argument_errors():
    w = np.zeros((2, 3, 3, 3), np.float32)
    pid = np.zeros((2, 3), np.uint8); conn = np.ones((2, 3), np.uint8)
    ok = np.array([0x03A], np.uint16)
    for table in (np.array([0], np.uint16), np.array([0x200], np.uint16)):
        with pytest.raises(P.PconvError) as e:
            P.pconv_pack(w, pid, conn, table, host_only=True)
        assert e.value.status == P.INVALID_ARG and "mask" in str(e.value)
    bad = pid.copy(); bad[1, 2] = 1
    with pytest.raises(P.PconvError) as e:
        P.pconv_pack(w, bad, conn, ok, host_only=True)
    assert e.value.status == P.INVALID_ARG and "f=1, c=2" in str(e.value)
    conn2 = conn.copy(); conn2[1, 2] = 0                    # same id on a removed kernel is fine
    P.pconv_pack(w, bad, conn2, ok, host_only=True).free()
    with pytest.raises(P.PconvError):
        P.pconv_pack(w, pid, conn, np.zeros(17, np.uint16) + 0x3A, host_only=True)
    L = P.lib()
    out = C.c_void_p()
    assert L.pconv_debug_pack_host(None, pid.ctypes.data, conn.ctypes.data, ok.ctypes.data, 1, 2, 3, 0,
                                   C.byref(out)) == P.INVALID_ARG
    assert L.pconv_debug_pack_host(w.ctypes.data, pid.ctypes.data, conn.ctypes.data, ok.ctypes.data, 1, 0, 3,
                                   0, C.byref(out)) == P.INVALID_ARG
    assert L.pconv_debug_pack_host(w.ctypes.data, pid.ctypes.data, conn.ctypes.data, ok.ctypes.data, 1, 2, 3,
                                   7, C.byref(out)) == P.INVALID_ARG
    L.pconv_free(None)                                      # NULL-safe


def test_host_only_handle_rejects_compute_and_policy_checks():
    w = np.ones((2, 3, 3, 3), np.float32)
    h = P.pconv_pack(w, np.zeros((2, 3), np.uint8), np.ones((2, 3), np.uint8),
                     np.array([0x03A], np.uint16), host_only=True)
    with pytest.raises(P.PconvError) as e:
        P.pconv_conv2d(h, 64, 128, 0, 1, 4, 4)
    assert e.value.status == P.INVALID_ARG
    for args in [dict(n=0), dict(h_in=0), dict(stride=3), dict(pad=0)]:
        kw = dict(n=1, h_in=4, w_in=4, stride=1, pad=1); kw.update(args)
        with pytest.raises(P.PconvError) as e:
            P.pconv_conv2d(h, 64, 128, 0, **kw)
        assert e.value.status == P.INVALID_ARG
    with pytest.raises(P.PconvError):
        P.pconv_conv2d(h, 64, 64, 0, 1, 4, 4)               # aliasing
    with pytest.raises(P.PconvError):
        P.pconv_set_kernel_policy(9)
    P.pconv_set_kernel_policy(0)
    h.free()


def test_blocks_are_a_balanced_deal_of_all_filters():
    """Workload balance of the tiled stream: every filter in exactly one slot, record counts add up,
    and inside every workgroup (16 blocks) no exchange of two filters between blocks lowers
    sum_b [ sum_j L(b,j)^2 + (sum_j L(b,j))^2 / J ]  (L = records of block b in chunk j),
    which is what the packer's local search minimises."""
    for seed, (f, c) in enumerate([(64, 64), (96, 40), (130, 23), (7, 9)]):
        spec = LayerSpec(f"bal{seed}", 1, c, f, 8, 8, num_patterns=12, pattern_dist="uniform",
                         keep_div=3.0, count_dist="bernoulli")
        L = make_layer(spec, 4000 + seed)
        h = P.pconv_pack(L["w"], L["pattern_id"], L["conn"], L["table"], "f32", host_only=True)
        slot_filter, records = P.pconv_debug_export_blocks(h)
        h.free()
        used = slot_filter[slot_filter >= 0]
        assert sorted(used.tolist()) == list(range(f))
        conn = L["conn"].astype(bool)
        J = records.shape[1]
        cpad = J * 8
        per_filter = np.zeros((f, J), np.int64)      # one record per kept kernel: all 12 masks are codes
        for j in range(J):
            per_filter[:, j] = conn[:, 8 * j:min(8 * j + 8, c)].sum(axis=1)
        want = np.zeros_like(records, dtype=np.int64)
        for b in range(slot_filter.shape[0]):
            for flt in slot_filter[b]:
                if flt >= 0:
                    want[b] += per_filter[flt]
        assert np.array_equal(records.astype(np.int64), want)

        def cost(load):                               # times J, in integers
            return int((load ** 2).sum() * J + (load.sum(axis=1) ** 2).sum())
        nb = slot_filter.shape[0]
        for g0 in range(0, nb, 16):
            blocks = range(g0, min(g0 + 16, nb))
            load = want[g0:g0 + 16].copy()
            base = cost(load)
            slots = [(b, s) for b in blocks for s in range(4)]
            for ia, (ba, sa) in enumerate(slots):
                for (bb, sb) in slots[ia + 1:]:
                    if ba == bb:
                        continue
                    fa, fb = slot_filter[ba, sa], slot_filter[bb, sb]
                    ca = per_filter[fa] if fa >= 0 else np.zeros(J, np.int64)
                    cb = per_filter[fb] if fb >= 0 else np.zeros(J, np.int64)
                    trial = load.copy()
                    trial[ba - g0] += cb - ca
                    trial[bb - g0] += ca - cb
                    assert cost(trial) >= base, (seed, ba, sa, bb, sb)
