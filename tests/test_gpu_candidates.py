"""Every launch configuration the tuner may adopt, against the CPU oracle.

xl_tune picks a block's configuration (kernel variant, tile, workgroup size, wave layout, chunk length,
output-channel split) by timing, so which one a benchmark run ends up with is not fixed.  Paper
section 3.2: the tuner must only change speed, never results.  Here every candidate of every launch of
configs 3, 4 and 5 is forced in turn (xl_plan_select_candidate) at the benchmark's full sizes and its
output compared element by element with the oracle: |g - o| <= 1e-4 + 1e-4 |o|.  Config 5 is checked block
by block (each fusion block cut out of the network with its real shapes and batch; the candidate lists
are the network plan's own, see test_blocks_cut_out_of_config5_plan_like_the_network_itself), so that
an error in one block is not averaged away by the layers after it.
"""
import numpy as np
import pytest

import xl_workloads as W
from oracle import xlo

pytestmark = pytest.mark.gpu

ATOL = 1e-4
RTOL = 1e-4


def check_on_device(torch, y, ref, what):
    """The comparison of test_gpu_parity.check, evaluated on the device (the outputs are up to 100 MB)."""
    assert y.shape == ref.shape, what
    if not bool(torch.isfinite(y).all()):
        raise AssertionError(f"{what}: non-finite output")
    err = (y.double() - ref.double()).abs()
    excess = err - (ATOL + RTOL * ref.double().abs())
    if bool((excess > 0).any()):
        idx = int(excess.argmax())
        raise AssertionError(f"{what}: {int((excess > 0).sum())} of {y.numel()} elements off; worst at flat index {idx}: "
                             f"gpu {float(y.flatten()[idx])!r} oracle {float(ref.flatten()[idx])!r}")


def run_every_candidate(wl, precision=0):
    import torch
    from paper_2007_06000_amd.session import Session
    x, params = W.make_tensors(wl)
    ref = torch.from_numpy(xlo.forward(wl, x, params)).cuda()
    s = Session(wl, x, params, precision=precision)
    total = 0
    for fused in (True, False):
        for launch in range(s.plan.num_launches(fused)):
            n = s.plan.num_candidates(fused, launch)
            for c in range(n):
                s.plan.select_candidate(fused, launch, c)
                info = s.plan.candidate_info(fused, launch)
                assert info["candidate"] == c
                what = (f"{wl.name} fused={fused} launch={launch} candidate={c}/{n} variant={info['variant']} "
                        f"tile={info['tile_h']}x{info['tile_w']} threads={info['threads']} csplit={info['cout_split']} "
                        f"waves={info['waves_cout_1']}/{info['waves_cout_2']} chunk={info['chunk_channels']} lds={info['lds_bytes']}")
                print("[case]", what, flush=True)
                s.y.fill_(float("nan"))
                s.run(fused)
                torch.cuda.synchronize()
                check_on_device(torch, s.y, ref, what)
                total += 1
            s.plan.select_candidate(fused, launch, 0)
    return total


@pytest.mark.parametrize("cfg", [3, 4])
def test_every_candidate_of_the_block_configs(cfg):
    assert run_every_candidate(W.config(cfg)) > 64


CFG5 = W.config(5)


@pytest.mark.parametrize("group", range(len(CFG5.groups)), ids=lambda g: CFG5.layers[CFG5.groups[g].layers[0]].name)
def test_every_candidate_of_every_block_of_config5(group):
    run_every_candidate(W.subgraph(CFG5, group))


def test_every_candidate_of_the_last_convolution_without_the_mean():
    """conv10 of config 5 on its own: the block above ends in a mean over the image, which would dilute a
    wrong pixel; the layer's own output shows it."""
    run_every_candidate(W.single_conv(64, 512, 13, 13, 1000, 1, seed=1040, dist="relu_normal"))


@pytest.mark.parametrize("cfg,kw", [(3, {}), (4, {"n": 8})])
def test_every_candidate_with_split_bf16_operands(cfg, kw):
    run_every_candidate(W.config(cfg, **kw), precision=1)


def test_merge_block_with_a_projection_shortcut():
    """The shortcut of a residual block may be any tensor produced before the block (here a 1x1 projection
    of the block input), not only the block input itself."""
    from test_gpu_parity import run_both
    wl = W.merge_residual_projection()
    out, ref, s = run_both(wl)
    assert s.plan.num_launches(True) == 2 and s.plan.num_launches(False) == 4
    run_both(wl, tune=True)


@pytest.mark.parametrize("cfg,kw", [(3, {}), (4, {"n": 4}), (5, {"n": 4})])
def test_blocks_switched_to_layer_by_layer_execution(cfg, kw):
    """xl_plan_set_block_fused: any mix of fused blocks and blocks run layer by layer gives the network's result
    (paper section 3.2: the tuner only changes speed)."""
    import torch
    from paper_2007_06000_amd.session import Session
    wl = W.config(cfg, **kw)
    x, params = W.make_tensors(wl)
    ref = torch.from_numpy(xlo.forward(wl, x, params)).cuda()
    s = Session(wl, x, params)
    ng = s.plan.num_groups
    for name, off in (("all", set(range(ng))), ("even", set(range(0, ng, 2))), ("odd", set(range(1, ng, 2))), ("none", set())):
        for g in range(ng):
            s.plan.set_block_fused(g, g not in off)
        what = f"{wl.name} layer-by-layer blocks: {name} launches={s.plan.num_launches(True)}"
        print("[case]", what, flush=True)
        s.y.fill_(float("nan"))
        s.run(True)
        torch.cuda.synchronize()
        check_on_device(torch, s.y, ref, what)
    assert s.plan.num_launches(True) == ng


def test_tuning_decides_fused_or_layer_by_layer_and_can_be_told_not_to():
    """After xl_tune a block runs layer by layer only if that measured faster; keep_blocks_fused = 1 pins every
    block to its kernel.  Either way the result is the oracle's."""
    import torch
    from paper_2007_06000_amd.session import Session
    wl = W.config(4, n=1)           # one image: 16 tiles cannot fill 256 compute units
    x, params = W.make_tensors(wl)
    ref = torch.from_numpy(xlo.forward(wl, x, params)).cuda()
    for keep in (0, 1):
        s = Session(wl, x, params, tune=True, keep_blocks_fused=keep)
        what = f"{wl.name} tuned keep_blocks_fused={keep} fused={[s.plan.block_is_fused(g) for g in range(s.plan.num_groups)]}"
        print("[case]", what, flush=True)
        if keep:
            assert s.plan.block_is_fused(0) and s.plan.num_launches(True) == 1
        else:
            assert s.plan.num_launches(True) in (1, s.plan.num_launches(False))
        s.y.fill_(float("nan"))
        s.run(True)
        torch.cuda.synchronize()
        check_on_device(torch, s.y, ref, what)


@pytest.mark.parametrize("wl", [
    W.conv_pool_generic(3, 3, 37, 41, 24, 3, 0, 2, 3, 2, 0),                 # ragged tiles, Cout not a multiple of 16
    W.conv_pool_generic(2, 3, 33, 29, 20, 3, 1, 2, 3, 2, 0, relu=False),     # padded convolution, negative values reach the pooling
    W.conv_pool_generic(2, 1, 40, 40, 7, 3, 0, 2, 3, 2, 0),                  # one input channel, 7 output channels
    W.conv_pool_generic(1, 3, 11, 11, 5, 3, 2, 2, 3, 2, 0, bn=True),         # tiny image, padding 2, folded BN
    W.conv_pool_generic(5, 3, 64, 20, 33, 3, 0, 2, 3, 2, 0),                 # tall image: tiles of one column
], ids=lambda w: w.name)
def test_every_candidate_of_stem_shaped_blocks(wl):
    """3x3 stride-2 convolution -> 3x3 stride-2 max pooling on a few input channels: besides the general thin kernel
    these blocks have the one where a lane owns the 2x2 block of convolution outputs under a pooled pixel."""
    from paper_2007_06000_amd import binding as B
    p = B.Plan(wl)
    variants = {p.candidate_info(True, 0, c)["variant"] for c in range(p.num_candidates(True, 0))}
    assert variants & {140, 141}, variants
    assert variants - {140, 141}, variants
    run_every_candidate(wl)
