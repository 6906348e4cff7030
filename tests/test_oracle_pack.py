"""Pins for the oracle's reference packer (canonical filter-kernel-reorder layout)."""
import json
import os

import numpy as np
import pytest

import oracle
from pconv_inputs import (LayerSpec, base_seed, config_layers, make_layer, nnz_of_layer,
                          vgg16_conv_shapes)


def python_pack(w, pid, conn, table, wdtype="f32"):
    """Second, independent implementation of the layout (numpy sorts, no shared code)."""
    import torch
    f, c = pid.shape
    p = len(table)
    kept = conn != 0
    hist = np.stack([((pid == q) & kept).sum(axis=1) for q in range(p)], axis=1)
    kcnt = kept.sum(axis=1)
    keys = [np.arange(f)] + [-hist[:, q] for q in reversed(range(p))] + [-kcnt]
    perm = np.lexsort(keys)
    row_ptr = np.concatenate([[0], np.cumsum(kcnt[perm])])
    cin, vals = [], []
    for fi in perm:
        cs = np.nonzero(kept[fi])[0]
        order = np.lexsort((cs, pid[fi, cs]))
        for ch in cs[order]:
            cin.append(ch)
            m = int(table[pid[fi, ch]])
            for t in range(9):
                if (m >> t) & 1:
                    vals.append(w[fi, ch, t // 3, t % 3])
    vals = np.array(vals, np.float32)
    if wdtype == "bf16":
        vals = torch.from_numpy(vals).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    return dict(perm=perm.astype(np.uint16), row_ptr=row_ptr.astype(np.uint32),
                pat_cnt=hist[perm].astype(np.uint16), cin=np.array(cin, np.uint16), vals=vals)


def test_hand_worked_example(golden_dir):
    g = json.load(open(os.path.join(golden_dir, "pack_tiny.json")))
    conn = np.array(g["conn"], np.uint8); pid = np.array(g["pattern_id"], np.uint8)
    table = np.array(g["table"], np.uint16)
    f, c = conn.shape
    w = np.array([[[100 * fi + 10 * ci + t for t in range(9)] for ci in range(c)]
                  for fi in range(f)], np.float32).reshape(f, c, 3, 3)
    pk = oracle.pack(w, pid, conn, table)
    assert pk["perm"].tolist() == g["perm"]
    assert pk["row_ptr"].tolist() == g["row_ptr"]
    assert pk["pat_cnt"].tolist() == g["pat_cnt"]
    assert pk["cin"].tolist() == g["cin"]
    assert pk["vals"].tolist() == [float(v) for v in g["vals"]]


@pytest.mark.parametrize("cfg", [1, 2, 5])
@pytest.mark.parametrize("wdtype", ["f32", "bf16"])
def test_invariants_roundtrip_and_second_implementation(cfg, wdtype):
    spec = config_layers(cfg)[0]
    L = make_layer(spec, base_seed(cfg))
    w, pid, conn, table = L["w"].copy(), L["pattern_id"], L["conn"], L["table"]
    # special bit patterns that must survive a bit copy
    kf, kc = np.nonzero(conn)
    m0 = int(table[pid[kf[0], kc[0]]]); t0 = [t for t in range(9) if (m0 >> t) & 1]
    w[kf[0], kc[0], t0[0] // 3, t0[0] % 3] = np.float32(-0.0)
    w[kf[0], kc[0], t0[1] // 3, t0[1] % 3] = np.float32(1e-41)
    pk = oracle.pack(w, pid, conn, table, wdtype)
    f, c = pid.shape
    kcnt = (conn != 0).sum(axis=1)
    # bijection, counts, pointer consistency
    assert sorted(pk["perm"].tolist()) == list(range(f))
    assert pk["row_ptr"][0] == 0 and pk["row_ptr"][f] == int((conn != 0).sum())
    assert np.array_equal(np.diff(pk["row_ptr"].astype(np.int64)), kcnt[pk["perm"]])
    assert np.array_equal(pk["pat_cnt"].sum(axis=1), kcnt[pk["perm"]])
    assert len(pk["vals"]) == nnz_of_layer(L)
    # sort keys non-increasing along perm, ties broken by filter index
    keys = [(int(kcnt[fi]),) + tuple(int(v) for v in pk["pat_cnt"][i]) for i, fi in enumerate(pk["perm"])]
    for i in range(1, f):
        assert keys[i - 1] >= keys[i]
        if keys[i - 1] == keys[i]:
            assert pk["perm"][i - 1] < pk["perm"][i]
    # every kept (f, c) exactly once, ordered by (pattern, channel) inside a filter
    seen = set()
    for i, fi in enumerate(pk["perm"]):
        ks = range(int(pk["row_ptr"][i]), int(pk["row_ptr"][i + 1]))
        pc = [(int(pid[fi, pk["cin"][k]]), int(pk["cin"][k])) for k in ks]
        assert pc == sorted(pc)
        for _, ch in pc:
            assert conn[fi, ch] and (int(fi), ch) not in seen
            seen.add((int(fi), ch))
    assert len(seen) == int((conn != 0).sum())
    # round trip is bit exact
    wt = oracle.masked_weights(w, pid, conn, table, wdtype).astype(np.float32)
    back = oracle.unpack(pk, table, c, wdtype)
    assert np.array_equal(back.view(np.uint32), wt.view(np.uint32))
    # independent implementation agrees byte for byte
    ref = python_pack(w, pid, conn, table, wdtype)
    for k in ("perm", "row_ptr", "pat_cnt", "cin"):
        assert np.array_equal(pk[k], ref[k]), k
    assert pk["vals"].tobytes() == ref["vals"].tobytes()


def test_degenerate_filters_and_mixed_popcounts():
    rng = np.random.default_rng(3)
    table = np.array([0x1FF, 0x010, 0x03A, 0x145], np.uint16)   # 9, 1, 4 and 3 taps
    f, c = 6, 7
    w = rng.standard_normal((f, c, 3, 3)).astype(np.float32)
    pid = rng.integers(0, 4, (f, c)).astype(np.uint8)
    conn = rng.integers(0, 2, (f, c)).astype(np.uint8)
    conn[2] = 0          # a filter with no kernels
    conn[4] = 1          # a filter with every kernel
    pk = oracle.pack(w, pid, conn, table)
    ref = python_pack(w, pid, conn, table)
    for k in ("perm", "row_ptr", "pat_cnt", "cin", "vals"):
        assert np.array_equal(pk[k], ref[k]), k
    back = oracle.unpack(pk, table, c)
    wt = oracle.masked_weights(w, pid, conn, table).astype(np.float32)
    assert np.array_equal(back.view(np.uint32), wt.view(np.uint32))
    assert pk["perm"][0] == 4 and pk["perm"][-1] == 2


def test_workload_accounting():
    """4-tap tables store 4 weights per kept kernel (2.25x); VGG-16 dense conv = 15.35 GMAC."""
    spec = config_layers(2)[0]
    L = make_layer(spec, base_seed(2))
    assert nnz_of_layer(L) == 4 * int(L["conn"].sum())
    kept = L["conn"].sum(axis=1)
    assert abs(L["conn"].mean() - 1 / 3.6) < 0.01 and kept.min() >= 49 and kept.max() <= 93
    shapes = vgg16_conv_shapes()
    macs = sum(ci * co * 9 * s * s for ci, co, s, _ in shapes)
    assert abs(macs / 1e9 - 15.35) < 0.01
    assert len({(ci, co, s) for ci, co, s, _ in shapes}) == 9      # 9 unique of 13 layer sizes
    L5 = make_layer(config_layers(5)[0], base_seed(5))
    k5 = L5["conn"].sum(axis=1)
    assert abs(k5.mean() - 64) < 8 and k5.max() > 250 and k5.min() >= 1
