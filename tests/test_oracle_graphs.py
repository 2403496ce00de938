"""Graph-level pins: the five workloads' shapes, parameter and FLOP counts, and
the oracle's graph walk against an independent torch float64 evaluation."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import xl_workloads as W
from oracle import xlo


def torch_forward(wl, x, params):
    """Independent evaluation with library routines in float64 (cross-check only)."""
    t = {wl.input_id: torch.from_numpy(x).double()}
    for li, L in enumerate(wl.layers):
        if L.op == "conv":
            p = params[li]
            y = F.conv2d(t[L.inputs[0]], torch.from_numpy(p["w"]).double(), None, L.stride, L.pad, 1, L.groups)
            if p["scale"] is not None:
                y = y * torch.from_numpy(p["scale"]).double().view(1, -1, 1, 1)
            if p["shift"] is not None:
                y = y + torch.from_numpy(p["shift"]).double().view(1, -1, 1, 1)
            if L.relu:
                y = y.clamp_min(0)
            y = y.float().double()          # intermediates are stored as fp32
        elif L.op == "maxpool":
            y = F.max_pool2d(t[L.inputs[0]], L.k, L.stride, L.pad)
        elif L.op == "gap":
            y = t[L.inputs[0]].mean(dim=(2, 3), keepdim=True).float().double()
        elif L.op == "add":
            y = t[L.inputs[0]] + t[L.inputs[1]]
            if L.relu:
                y = y.clamp_min(0)
            y = y.float().double()
        elif L.op == "concat":
            y = torch.cat([t[L.inputs[0]], t[L.inputs[1]]], dim=1)
        t[L.out] = y
    return t[wl.output_id].float().numpy()


def test_config_shapes():
    assert W.config(1).shapes[-1] == (1, 16, 16, 16)
    assert W.config(2).shapes[-1] == (8, 64, 28, 28)
    assert W.config(3).shapes[-1] == (16, 128, 55, 55)
    assert W.config(4).shapes[-1] == (32, 64, 56, 56)
    wl = W.config(5)
    assert wl.shapes[wl.output_id] == (64, 1000, 1, 1)
    spatial = [wl.shapes[L.out][2] for L in wl.layers if L.op in ("conv", "maxpool") and L.name in
               ("conv1", "pool1", "pool2", "pool3")]
    assert spatial == [111, 55, 27, 13]                       # 224 -> 111 -> 55 -> 27 -> 13
    assert sum(1 for g in wl.groups if g.mode == "split") == 8   # 8 mode-b blocks (paper section 4.2)


def test_config5_parameter_and_flop_count():
    wl = W.config(5)
    assert W.count_params(wl) == 1_235_496                   # SqueezeNet v1.1 with 1000 classes
    per_image = W.count_flops(wl) / wl.batch
    assert abs(per_image / 1e6 - 698.3) < 0.1


def test_flops_of_block_configs():
    assert W.count_flops(W.config(1)) == 2 * 2 * 16 * 16 * 16 * 16 * 9
    assert abs(W.count_flops(W.config(2)) / 1e6 - 205.5) < 0.1
    assert abs(W.count_flops(W.config(3)) / 1e9 - 1.140) < 0.001
    assert abs(W.count_flops(W.config(4)) / 1e9 - 14.80) < 0.01


def test_tensor_recipes():
    x, p = W.make_tensors(W.config(1))
    assert x.dtype == np.float32 and 0.0 <= x.min() and x.max() < 1.0
    w = p[0]["w"]
    assert abs(w.std() - np.sqrt(2 / 144)) < 0.01 and p[0]["scale"] is None
    assert abs(p[0]["shift"].std() - 0.01) < 0.008
    x4, p4 = W.make_tensors(W.config(4, n=2))
    assert x4.min() == 0.0 and (x4 == 0).mean() > 0.4        # ReLU'd N(0,1)
    assert abs(p4[0]["scale"].mean() - 1.0) < 0.05 and abs(p4[0]["shift"].std() - 0.1) < 0.04
    xa, _ = W.make_tensors(W.config(3, n=1))
    xb, _ = W.make_tensors(W.config(3, n=1))
    np.testing.assert_array_equal(xa, xb)                     # seeded


@pytest.mark.parametrize("cfg,kw", [
    (1, {}),
    (2, {"n": 2}),
    (3, {"n": 1, "hw": 19}),
    (4, {"n": 1, "hw": 14, "c": 16}),
    (5, {"n": 1, "hw": 63, "classes": 24}),
])
def test_graph_walk_against_torch(cfg, kw):
    wl = W.config(cfg, **kw)
    x, params = W.make_tensors(wl)
    got = xlo.forward(wl, x, params)
    ref = torch_forward(wl, x, params)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=2e-6, atol=2e-6)


def test_merge_block_is_residual_formula():
    """Config 4's block, written out: relu(bn2(conv2(relu(bn1(conv1 x)))) + x)."""
    wl = W.config(4, n=1, hw=9, c=8)
    x, p = W.make_tensors(wl)
    y1 = xlo.conv2d(x, p[0]["w"], 1, 1, 1, p[0]["scale"], p[0]["shift"], True)
    y2 = xlo.conv2d(y1, p[1]["w"], 1, 1, 1, p[1]["scale"], p[1]["shift"], False)
    ref = np.maximum(y2 + x, 0)
    np.testing.assert_array_equal(xlo.forward(wl, x, p), ref)


def test_split_block_concat_order():
    """expand1x1 fills channels [0,E), expand3x3 fills [E,2E)."""
    wl = W.config(3, n=1, hw=7, cin=8, s=4, e=6)
    x, p = W.make_tensors(wl)
    t = xlo.forward(wl, x, p, keep_all=True)
    sq = xlo.conv2d(x, p[0]["w"], 1, 0, 1, None, p[0]["shift"], True)
    np.testing.assert_array_equal(t[wl.output_id][:, :6], xlo.conv2d(sq, p[1]["w"], 1, 0, 1, None, p[1]["shift"], True))
    np.testing.assert_array_equal(t[wl.output_id][:, 6:], xlo.conv2d(sq, p[2]["w"], 1, 1, 1, None, p[2]["shift"], True))
