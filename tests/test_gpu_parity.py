"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element, on the same seeded inputs.  Bar: |g - o| <= 1e-4 + 1e-4 |o| in fp32
for every element, fused and unfused."""
import numpy as np
import pytest

import xl_workloads as W
from oracle import xlo

pytestmark = pytest.mark.gpu

ATOL = 1e-4
RTOL = 1e-4


def check(got: np.ndarray, ref: np.ndarray, what: str):
    assert got.shape == ref.shape, what
    assert np.isfinite(got).all(), f"{what}: non-finite output"
    err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
    bound = ATOL + RTOL * np.abs(ref.astype(np.float64))
    bad = err > bound
    if bad.any():
        idx = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {bad.sum()} of {bad.size} elements off; worst at {idx}: "
                             f"gpu {got[idx]!r} oracle {ref[idx]!r}")
    return float(err.max())


_REF = {}       # oracle outputs of the full-size configs, computed once per test session (seeded inputs)


def oracle_output(wl, x, params):
    key = (wl.name, tuple(wl.shapes[0]), len(wl.layers), wl.seed)
    if int(np.prod(wl.shapes[0])) < (1 << 20):
        return xlo.forward(wl, x, params)
    if key not in _REF:
        _REF[key] = xlo.forward(wl, x, params)
    return _REF[key]


def run_both(wl, **options):
    from paper_2007_06000_amd.session import Session
    x, params = W.make_tensors(wl)
    ref = oracle_output(wl, x, params)
    s = Session(wl, x, params, **options)
    out = {}
    for fused in (True, False):
        print(f"[case] {wl.name} shapes={wl.shapes[0]} fused={fused} opts={options}", flush=True)
        got = s.output(fused)
        out[fused] = got
        check(got, ref, f"{wl.name} fused={fused}")
    return out, ref, s


SMALL = [
    (1, {}),
    (1, {"hw": 13}),
    (2, {"n": 2, "hw": 20}),
    (2, {"n": 1, "hw": 15, "c": 24}),
    (3, {"n": 2, "hw": 19}),
    (3, {"n": 1, "hw": 11, "cin": 40, "s": 16, "e": 64}),
    (3, {"n": 1, "hw": 13, "cin": 72, "s": 48, "e": 96}),
    (4, {"n": 2, "hw": 17, "c": 32}),
    (4, {"n": 1, "hw": 9, "c": 64}),
    (5, {"n": 2, "hw": 63, "classes": 40}),
]


@pytest.mark.parametrize("cfg,kw", SMALL)
def test_small_and_ragged(cfg, kw):
    run_both(W.config(cfg, **kw))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_block_configs_full_size(cfg):
    run_both(W.config(cfg))


def test_config5_full_size():
    run_both(W.config(5))


@pytest.mark.parametrize("cfg,kw,tile", [
    (1, {}, (4, 4)), (1, {}, (16, 16)), (1, {}, (5, 7)),
    (3, {"n": 2, "hw": 19}, (13, 19)), (3, {"n": 2, "hw": 19}, (5, 8)), (3, {"n": 2, "hw": 19}, (3, 19)),
    (4, {"n": 2, "hw": 17, "c": 32}, (6, 6)), (4, {"n": 2, "hw": 17, "c": 32}, (14, 14)),
    (2, {"n": 2, "hw": 20}, (2, 10)), (2, {"n": 2, "hw": 20}, (5, 5)),
])
def test_tile_choice_does_not_change_the_result(cfg, kw, tile):
    """Fusion order / tile size must not change the math (beyond fp32 reassociation)."""
    run_both(W.config(cfg, **kw), force_tile_h=tile[0], force_tile_w=tile[1])


@pytest.mark.parametrize("split", [1, 2, 4])
def test_cout_split(split):
    run_both(W.config(3, n=1, hw=13, cin=64, s=32, e=128), force_cout_split=split)


def test_prezeroed_intermediate_border():
    """Bias +1 everywhere: halo positions outside the image must reach layer 2 as 0, not relu(bias)."""
    wl = W.config(1)
    x, params = W.make_tensors(wl)
    for p in params.values():
        p["shift"] = np.ones_like(p["shift"])
    ref = xlo.forward(wl, x, params)
    from paper_2007_06000_amd.session import Session
    for tile in ((16, 16), (4, 8), (7, 5)):
        s = Session(wl, x, params, force_tile_h=tile[0], force_tile_w=tile[1])
        check(s.output(True), ref, f"border tile={tile}")


def test_batch_independence_bitwise():
    wl3 = W.config(3, n=3, hw=19)
    x, params = W.make_tensors(wl3)
    from paper_2007_06000_amd.session import Session
    full = Session(wl3, x, params, force_tile_h=7, force_tile_w=7).output(True)
    wl1 = W.config(3, n=1, hw=19)
    for n in range(3):
        one = Session(wl1, x[n:n + 1], params, force_tile_h=7, force_tile_w=7).output(True)
        np.testing.assert_array_equal(one[0], full[n])


def test_single_convs():
    for wl in (W.single_conv(2, 3, 31, 31, 64, 3, stride=2, pad=0),
               W.single_conv(1, 512, 13, 13, 1000, 1),
               W.single_conv(2, 20, 9, 11, 24, 3, stride=1, pad=1, bias=False, bn=True, relu=False),
               W.single_conv(1, 8, 7, 7, 8, 1, relu=False)):
        run_both(wl)


@pytest.mark.parametrize("cfg,kw", [(1, {}), (2, {"n": 2, "hw": 20}), (3, {}), (4, {"n": 2, "hw": 28}),
                                    (5, {"n": 2, "hw": 95, "classes": 40})])
def test_tuned_plans_match_the_oracle(cfg, kw):
    """xl_tune swaps in other candidates (tiles, workgroup sizes, splits): results must not change."""
    from paper_2007_06000_amd.session import Session
    wl = W.config(cfg, **kw)
    x, params = W.make_tensors(wl)
    ref = xlo.forward(wl, x, params)
    s = Session(wl, x, params, tune=True)
    for fused in (True, False):
        print(f"[case] tuned {wl.name} fused={fused}", flush=True)
        check(s.output(fused), ref, f"tuned {wl.name} fused={fused}")
    q = s.plan.query(0)
    assert q["lds_bytes"] <= 160 * 1024 and q["workgroups"] > 0


@pytest.mark.parametrize("cfg", [4, 5])
def test_full_size_configs_with_the_plans_the_benchmark_times(cfg):
    """bench.py times tuned plans at the full benchmark sizes: the same launch configuration, every element."""
    run_both(W.config(cfg), tune=True)


@pytest.mark.parametrize("shape", [
    dict(n=3, cin=40, h=13, w=13, c1=100, k1=1, p1=0, s1=1),            # pointwise, ragged channels: one row of 169 pixels
    dict(n=2, cin=24, h=9, w=11, c1=70, k1=3, p1=1, s1=1, bn=True),     # 3x3 with folded batch-norm
    dict(n=2, cin=16, h=7, w=5, c1=33, k1=3, p1=0, s1=1, relu=False),   # no activation: negative values in the mean
    dict(n=1, cin=8, h=1, w=1, c1=16, k1=1, p1=0, s1=1),                # one pixel
])
def test_conv_then_global_average_pooling(shape):
    """Straight block conv -> global average pooling: the mean is formed inside the convolution kernel."""
    out, ref, s = run_both(W.conv_gap_generic(**shape))
    assert s.plan.num_launches(True) == 1 and s.plan.num_launches(False) == 2


@pytest.mark.parametrize("wl", [
    W.single_conv(2, 64, 13, 13, 100, 1),               # one row of 169 pixels: width not a multiple of 4
    W.single_conv(3, 32, 27, 27, 48, 1, bn=True),       # 729 pixels: several tiles per image, ragged last one
    W.single_conv(1, 16, 5, 7, 8, 1),
    W.single_conv(2, 128, 1, 1, 64, 1),                 # a single pixel
    W.straight_generic(2, 64, 13, 11, 32, 1, 0, 1, 48, 3, 1, 1),        # 1x1 -> 3x3: halo rows/columns outside the image
    W.straight_generic(1, 48, 9, 30, 16, 1, 0, 1, 24, 3, 1, 1, bn1=True),
    W.config(3, n=2, hw=21, cin=64, s=16, e=32),                        # fire block, image not a multiple of any tile
], ids=lambda w: w.name)
def test_pointwise_first_layers_with_whole_k_steps_of_channels(wl):
    """1x1 first layers whose channel count is a multiple of the K step may use the planar input
    staging (LDS-direct loads); the cases cover unaligned rows, ragged tiles and image borders."""
    for tune in (False, True):
        from paper_2007_06000_amd.session import Session
        x, params = W.make_tensors(wl)
        ref = xlo.forward(wl, x, params)
        s = Session(wl, x, params, tune=tune)
        for fused in (True, False):
            print(f"[case] {wl.name} tune={tune} fused={fused}", flush=True)
            check(s.output(fused), ref, f"{wl.name} tune={tune} fused={fused}")


@pytest.mark.parametrize("wl", [
    W.straight_generic(2, 192, 28, 28, 16, 1, 0, 1, 32, 5, 2, 1),       # paper Table 1, a.1 (inception 5x5 branch), batch 2
    W.straight_generic(1, 20, 11, 9, 24, 1, 0, 1, 40, 5, 2, 1, bn2=True),
    W.straight_generic(1, 8, 12, 12, 12, 3, 1, 1, 20, 5, 0, 1),         # 3x3 -> 5x5 without padding
    W.single_conv(2, 6, 13, 10, 35, 5, stride=1, pad=2),
    W.single_conv(1, 3, 17, 17, 8, 5, stride=2, pad=2),
], ids=lambda w: w.name)
def test_five_by_five_filters(wl):
    run_both(wl)
    run_both(wl, tune=True)     # the tuner also tries the variants that stage a pointwise first layer's input as planes


@pytest.mark.parametrize("wl", [
    W.depthwise_pointwise(2, 16, 80, 80, 16),                                # paper Table 1, a.2, batch 2
    W.depthwise_pointwise(1, 10, 13, 9, 24, bn1=True),                       # channels not a multiple of 4
    W.depthwise_pointwise(2, 32, 17, 17, 40, s1=2, relu1=False),             # strided depthwise, negative intermediate
    W.depthwise_pointwise(1, 64, 14, 14, 64, k2=3, p2=1, bn2=True),          # depthwise -> 3x3: halo of the intermediate
    W.depthwise_pointwise(1, 3, 5, 5, 4, p1=0),
], ids=lambda w: w.name)
def test_depthwise_then_convolution(wl):
    out, ref, s = run_both(wl)
    assert s.plan.num_launches(True) == 1 and s.plan.num_launches(False) == 2


@pytest.mark.parametrize("wl", [
    W.merge_two_producers(2, 64, 56, 56, 256, 64),                           # paper Table 1, c.1, batch 2
    W.merge_two_producers(1, 24, 9, 11, 72, 40, bn=False),                   # ragged pixels and channels
    W.merge_two_producers(2, 16, 7, 7, 33, 20, relu_a=True, relu_sum=False), # activation on one producer, none on the sum
], ids=lambda w: w.name)
def test_merge_block_with_two_producers(wl):
    out, ref, s = run_both(wl)
    assert s.plan.num_launches(True) == 1 and s.plan.num_launches(False) == 4


@pytest.mark.parametrize("wl", [
    W.conv_pool_generic(3, 3, 37, 41, 24, 3, 0, 2, 3, 2, 0),            # stem-like: 3 channels, stride 2, ragged tiles
    W.conv_pool_generic(70, 3, 9, 9, 8, 3, 1, 1, 2, 2, 0),              # many tiny images: more tiles than resident workgroups
    W.conv_pool_generic(2, 8, 19, 23, 40, 3, 1, 1, 3, 2, 1, bn=True),   # padding on both layers
    W.conv_pool_generic(1, 16, 30, 30, 64, 1, 0, 1, 3, 2, 1),           # 1x1 first layer, whole reduction in one chunk
    W.conv_pool_generic(2, 5, 11, 7, 12, 3, 1, 1, 3, 1, 1, relu=False), # stride-1 pooling over negative values
], ids=lambda w: w.name)
def test_conv_then_max_pooling_shapes(wl):
    """conv -> maxpool blocks, among them first layers whose reduction fits one chunk (served by the
    kernel that walks a stream of tiles per workgroup)."""
    for tune in (False, True):
        from paper_2007_06000_amd.session import Session
        x, params = W.make_tensors(wl)
        ref = xlo.forward(wl, x, params)
        s = Session(wl, x, params, tune=tune)
        for fused in (True, False):
            print(f"[case] {wl.name} tune={tune} fused={fused}", flush=True)
            check(s.output(fused), ref, f"{wl.name} tune={tune} fused={fused}")


@pytest.mark.parametrize("wl", [
    W.split_fire_pool(),                                        # 27 -> 13, the shape between fire modules
    W.split_fire_pool(n=1, cin=40, hw=15, s=16, e=64),          # 15 -> 7
    W.split_fire_pool(n=2, cin=24, hw=14, s=8, e=16),           # last row and column feed no window
    W.split_fire_pool(n=1, cin=72, hw=12, s=48, e=96, pk=2, ps=2),
    W.split_fire_pool(n=3, cin=64, hw=55, s=16, e=64),          # config 5's fire3 + pool
    W.split_fire_pool(n=2, cin=32, hw=27, pp=1),                # padded pooling: windows start above / left of the image
    W.split_fire_pool(n=1, cin=40, hw=14, s=16, e=64, pp=1),    # ... and hang over its bottom / right edge
    W.split_fire_pool(n=2, cin=64, hw=13, s=48, e=96, pk=2, ps=2, pp=1),
])
def test_split_block_with_max_pooling(wl):
    run_both(wl)
    run_both(wl, tune=True)


def test_degenerate_shapes():
    """1x1 images, single channels, tiles larger than the image, odd sizes under stride 2."""
    for wl in (W.single_conv(1, 1, 1, 1, 1, 1),
               W.single_conv(3, 1, 5, 7, 1, 3, stride=1, pad=1),
               W.single_conv(2, 5, 9, 9, 3, 3, stride=2, pad=1),
               W.straight_generic(1, 3, 3, 3, 5, 3, 1, 1, 4, 3, 1, 1),
               W.straight_generic(2, 17, 6, 5, 33, 1, 0, 1, 9, 3, 1, 1, bn1=True),
               W.conv_pool_generic(1, 4, 7, 9, 6, 3, 1, 1, 3, 2, 0),
               W.conv_pool_generic(2, 3, 12, 12, 8, 3, 0, 2, 2, 2, 0, relu=False),
               W.config(3, n=1, hw=1, cin=8, s=16, e=32),
               W.config(4, n=1, hw=2, c=16)):
        run_both(wl)


def test_empty_batch_runs_nothing():
    import torch
    from paper_2007_06000_amd.session import Session
    wl = W.config(3, n=0)
    x, params = W.make_tensors(wl)
    s = Session(wl, x, params)
    s.run(True)
    s.run(False)
    torch.cuda.synchronize()
    assert s.y.numel() == 0
