"""GPU parity of the split-bf16 kernels (xl_options.precision = XL_PRECISION_BF16X3) against the fp64
CPU oracle: same bar as the fp32 kernels, |g - o| <= 1e-4 + 1e-4 |o| for every element."""
import numpy as np
import pytest

import xl_workloads as W
from test_gpu_parity import run_both, SMALL

pytestmark = pytest.mark.gpu

BF16X3 = 1


def run_split(wl, expect_split=True, **options):
    out, ref, s = run_both(wl, precision=BF16X3, **options)
    precisions = [s.plan.query(g)["precision"] for g in range(s.plan.num_groups)]
    if expect_split:
        assert BF16X3 in precisions, "no block of the plan runs a split-bf16 kernel"
    return out, ref, s


@pytest.mark.parametrize("cfg,kw", SMALL)
def test_small_and_ragged(cfg, kw):
    run_split(W.config(cfg, **kw))


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_block_configs_full_size(cfg):
    run_split(W.config(cfg))


def test_config5_full_size():
    run_split(W.config(5))


@pytest.mark.parametrize("cfg", [4, 5])
def test_full_size_configs_with_tuned_plans(cfg):
    run_split(W.config(cfg), expect_split=False, tune=True)


@pytest.mark.parametrize("cfg,kw", [(3, {}), (4, {"n": 2, "hw": 28}), (5, {"n": 2, "hw": 63, "classes": 40})])
def test_tuned_plans(cfg, kw):
    run_split(W.config(cfg, **kw), expect_split=False, tune=True)


@pytest.mark.parametrize("wl", [
    W.straight_generic(2, 40, 14, 14, 16, 1, 0, 1, 32, 5, 2, 1),
    W.conv_gap_generic(2, 24, 9, 9, 50, 1, 0, 1),
    W.conv_gap_generic(1, 19, 13, 13, 70, 3, 1, 1),
])
def test_other_structures(wl):
    run_split(wl)


@pytest.mark.parametrize("wl", [W.depthwise_pointwise(2, 16, 20, 20, 16), W.depthwise_pointwise(1, 10, 13, 9, 24, bn1=True),
                                W.merge_two_producers(2, h=14, w=14), W.merge_two_producers(1, c=24, h=9, w=11, cmid=40, cout=20),
                                W.split_fire_pool(), W.split_fire_pool(n=1, cin=40, hw=15, s=16, e=64)],
                         ids=lambda w: w.name)
def test_depthwise_two_producer_and_pooled_split_blocks(wl):
    out, ref, s = run_split(wl)
    assert s.plan.query(0)["precision"] == BF16X3
    run_split(wl, expect_split=False, tune=True)        # the tuner may keep an fp32 kernel where it measures faster


def test_large_and_tiny_magnitudes():
    # operands far from 1: the split keeps the relative error of each product
    wl = W.config(4, n=1, hw=12, c=32)
    x, params = W.make_tensors(wl)
    from oracle import xlo
    from paper_2007_06000_amd.session import Session
    x = (x * 1e3).astype(np.float32)
    ref = xlo.forward(wl, x, params)
    s = Session(wl, x, params, precision=BF16X3)
    got = s.output(True)
    err = np.abs(got.astype(np.float64) - ref)
    assert (err <= 1e-4 * np.abs(ref).max()).all()
