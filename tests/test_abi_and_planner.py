"""CPU-side checks: the C-ABI library loads and exports every declared symbol;
the planner's halo arithmetic, tuner search space, traffic accounting and error
paths (no device needed: plans are made for a nominal gfx950)."""
import ctypes
import os
import re

import pytest

import xl_workloads as W
from paper_2007_06000_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def golden(name):
    rows = []
    for ln in open(os.path.join(ROOT, "tests", "golden", name)):
        ln = ln.split("#")[0].strip()
        if ln:
            rows.append(ln.split())
    return rows


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "xl.h")).read()
    declared = set(re.findall(r"\b(xl_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.xl_version().startswith("xl ")
    assert B.xl_strerror(B.XL_E_LDS_BUDGET) and B.xl_strerror(0) == "ok"


def test_tuner_search_space_matches_paper_example():
    """Section 3.2: output size (12,12) -> {(4,3), (2,6), (3,4), (6,2)} as (tile, grid)."""
    want = {(int(a), int(b)) for a, b in golden("tuner_example.txt")}
    assert set(B.xl_tuner_candidates(12)) == want
    # a prime size is searched on the next larger non-prime
    assert set(B.xl_tuner_candidates(13)) == {(2, 7), (7, 2)}
    assert (14, 4) in B.xl_tuner_candidates(55) or (5, 11) in B.xl_tuner_candidates(55)


def test_halo_arithmetic():
    assert B.xl_required_extent(14, 3, 1) == 16
    assert B.xl_required_extent(14, 1, 1) == 14          # filter size 1: no redundant data (section 3.2)
    assert B.xl_required_extent(7, 3, 2) == 15
    # section 3.2 example: 3x3 tiles on 2x2 blocks over a 5x5 map store 36 elements for 25 unique
    tile = 3
    assert 4 * tile * tile == 36 and (2 * tile - 1) ** 2 == 25


@pytest.mark.parametrize("row", golden("table2_store_transactions.txt"))
def test_store_counts_follow_paper_table2(row):
    """Table 2: unfused stores = every layer output, fused stores = block output only
    (the paper's counters report 2 and 4 floats per transaction respectively)."""
    case, cin, h, w, c1, k1, p1, c2, k2, p2, ours, cudnn = row[0], *map(int, row[1:])
    wl = W.straight_generic(1, cin, h, w, c1, k1, p1, 1, c2, k2, p2, 1) if case != "b.1" else W.config(3, n=1, cin=cin, hw=h, s=c1, e=c2)
    p = B.Plan(wl)
    q = p.query(0)
    assert q["stores_unfused"] == 2 * cudnn
    assert q["stores_fused"] == 4 * ours


def test_store_counts_of_the_depthwise_case_of_table2():
    """Table 2, a.2 (depthwise 3x3 -> pointwise on [16,80,80]): 25600 fused vs 102400 per-layer
    transactions, i.e. 4 and 2 floats per transaction over 102400 and 204800 stored elements."""
    q = B.Plan(W.depthwise_pointwise(1, 16, 80, 80, 16)).query(0)
    assert q["stores_fused"] == 4 * 25600 and q["stores_unfused"] == 2 * 102400
    assert q["mode"] == B.XL_STRAIGHT and q["mid_h"] == q["tile_h"] and q["in_h"] == q["tile_h"] + 2


def test_grouped_convolutions_other_than_depthwise_are_rejected():
    wl = W.single_conv(1, 8, 9, 9, 8, 3, pad=1)
    wl.layers[0].groups = 2
    with pytest.raises(B.XlError) as e:
        B.Plan(wl)
    assert e.value.status == B.XL_E_UNSUPPORTED


def test_two_producer_merge_block_plans_as_one_launch():
    """Table 1, c.1: {1x1 64->256, 1x1 64->256} -> add -> 1x1 256->64 on [64,56,56]."""
    p = B.Plan(W.merge_two_producers(1))
    q = p.query(0)
    assert q["mode"] == B.XL_MERGE and q["nlayers"] == 4 and p.num_launches(True) == 1
    assert q["stores_fused"] == 64 * 56 * 56 and q["stores_unfused"] == (3 * 256 + 64) * 56 * 56
    assert q["bytes_fused"] < q["bytes_unfused"] / 5


def test_algorithmic_traffic_of_the_block_configs():
    want = {1: (51.3e3, 84.1e3), 2: (8.05e6, 20.89e6), 3: (43.41e6, 52.71e6), 4: (51.68e6, 180.13e6)}
    for cfg, (fused, unfused) in want.items():
        q = B.Plan(W.config(cfg)).query(0)
        assert abs(q["bytes_fused"] - fused) / fused < 0.005
        assert abs(q["bytes_unfused"] - unfused) / unfused < 0.005
        assert q["bytes_fused"] < q["bytes_unfused"]
        assert q["lds_bytes"] <= 160 * 1024 and q["workgroups"] > 0


def test_config5_plan_has_eight_split_blocks_and_fewer_launches():
    p = B.Plan(W.config(5))
    modes = [p.query(g)["mode"] for g in range(p.num_groups)]
    assert modes.count(B.XL_SPLIT) == 8
    assert p.num_launches(True) < p.num_launches(False)
    assert p.workspace_bytes() > 0


def test_lds_budget_is_enforced():
    wl = W.config(4)
    with pytest.raises(B.XlError) as e:
        B.Plan(wl, lds_budget_bytes=16 * 1024)
    assert e.value.status == B.XL_E_LDS_BUDGET
    q = B.Plan(wl, lds_budget_bytes=100 * 1024).query(0)
    assert q["lds_bytes"] <= 100 * 1024


def test_forced_tile_and_redundancy():
    q = B.Plan(W.config(4), force_tile_h=14, force_tile_w=14).query(0)
    assert (q["tile_h"], q["tile_w"], q["mid_h"], q["mid_w"], q["in_h"], q["in_w"]) == (14, 14, 16, 16, 18, 18)
    assert abs(q["redundancy"] - 256 / 196) < 1e-9
    assert q["flops_executed"] >= q["flops"]


def test_error_paths():
    wl = W.config(1)
    wl.layers[0].groups = 4                  # grouped but not depthwise
    with pytest.raises(B.XlError) as e:
        B.Plan(wl)
    assert e.value.status == B.XL_E_UNSUPPORTED
    wl = W.config(1)
    wl.shapes[1] = (1, 16, 15, 16)
    with pytest.raises(B.XlError) as e:
        B.Plan(wl)
    assert e.value.status == B.XL_E_SHAPE
    wl = W.config(1)
    wl.groups[0] = W.Group("merge", (0, 1))
    with pytest.raises(B.XlError) as e:
        B.Plan(wl)
    assert e.value.status == B.XL_E_UNSUPPORTED
    wl = W.config(2)
    wl.groups = [W.Group("single", (0,)), W.Group("straight", (0, 1))]
    with pytest.raises(B.XlError) as e:
        B.Plan(wl)
    assert e.value.status == B.XL_E_GRAPH


def test_oversized_tensors_are_rejected_cleanly():
    wl = W.single_conv(1, 8, 20000, 20000, 8, 1)            # 3.2e9 elements per image
    with pytest.raises(B.XlError) as e:
        B.Plan(wl)
    assert e.value.status == B.XL_E_UNSUPPORTED


def test_global_average_pooling_block_needs_the_image_in_one_tile():
    ok = B.Plan(W.conv_gap_generic(2, 16, 13, 13, 64, 1, 0, 1))
    q = ok.query(0)
    assert q["tiles_y"] * q["tiles_x"] == 1 and q["stores_fused"] == 2 * 64
    assert q["stores_unfused"] == 2 * 64 * 169 + 2 * 64
    with pytest.raises(B.XlError) as e:                         # 112 x 112 pixels do not fit one workgroup
        B.Plan(W.conv_gap_generic(1, 16, 112, 112, 64, 1, 0, 1))
    assert e.value.status == B.XL_E_UNSUPPORTED


def test_empty_batch_plans():
    p = B.Plan(W.config(3, n=0))
    assert p.query(0)["workgroups"] == 0


def test_paper_tuner_only_restricts_tiles():
    """With paper_tuner_only the tile is one of the square common-factor tiles of section 3.2."""
    wl = W.config(4, n=4)                       # 56 = 2*2*2*7
    q = B.Plan(wl, paper_tuner_only=1).query(0)
    allowed = {t for t, g in B.xl_tuner_candidates(56)}
    assert q["tile_h"] == q["tile_w"] and q["tile_h"] in allowed


def test_precision_option_selects_split_bf16_kernels_where_they_exist():
    q = B.Plan(W.config(4)).query(0)
    assert q["precision"] == 0
    q = B.Plan(W.config(4), precision=1).query(0)
    assert q["precision"] == 1 and q["chunk_channels"] % 16 == 0     # a K step covers 16 or 32 channels
    # every block kind has split-bf16 variants (a depthwise first layer itself stays on the vector ALU in fp32)
    for wl in (W.depthwise_pointwise(1, 16, 80, 80, 16), W.merge_two_producers(1), W.split_fire_pool(), W.config(2), W.config(3)):
        assert B.Plan(wl, precision=1).query(0)["precision"] == 1
    with pytest.raises(B.XlError):
        B.Plan(W.config(4), precision=2)


def test_split_bf16_error_model():
    """x = hi + lo + r with hi = bf16(x), lo = bf16(x - hi) (round to nearest even), and
    a*b ~ hi*hi + hi*lo + lo*hi: the part left out (lo*lo and the two r terms, each at most
    2^-16 |a||b|) stays below 3 * 2^-16 |a||b| per product, which over
    the reductions of the benchmark configs (up to 9 * 512 terms of random sign) is far inside the
    1e-4 parity tolerance."""
    import numpy as np

    def bf16(x):
        u = x.astype(np.float32).view(np.uint32).astype(np.uint64)
        u = (u + 0x7fff + ((u >> 16) & 1)) & 0xffff0000
        return u.astype(np.uint32).view(np.float32)

    rng = np.random.default_rng(5)
    a = (rng.standard_normal(1 << 16) * np.exp(rng.uniform(-20, 20, 1 << 16))).astype(np.float32)
    b = (rng.standard_normal(1 << 16) * np.exp(rng.uniform(-20, 20, 1 << 16))).astype(np.float32)
    ah, bh = bf16(a), bf16(b)
    al, bl = bf16(a - ah), bf16(b - bh)
    assert (np.abs(a - ah) <= 2.0 ** -8 * np.abs(a)).all() and (np.abs(al) <= 2.0 ** -8 * np.abs(a)).all()
    approx = ah.astype(np.float64) * bh + ah.astype(np.float64) * bl + al.astype(np.float64) * bh
    exact = a.astype(np.float64) * b
    assert (np.abs(approx - exact) <= 3 * 2.0 ** -16 * np.abs(exact)).all()
    # a reduction of the size of config 4's (64 channels x 9 taps), unit-variance operands scaled like the workloads
    K = 576
    x = rng.standard_normal((256, K)).astype(np.float32)
    w = (rng.standard_normal((K, 64)) / np.sqrt(K)).astype(np.float32)
    xh, wh = bf16(x), bf16(w)
    xl, wl = bf16(x - xh), bf16(w - wh)
    y3 = xh.astype(np.float64) @ wh + xh.astype(np.float64) @ wl + xl.astype(np.float64) @ wh
    y = x.astype(np.float64) @ w
    assert np.abs(y3 - y).max() < 2e-5      # a fifth of the absolute part of the tolerance


def test_split_block_followed_by_max_pooling_is_one_launch():
    wl = W.split_fire_pool(n=2, cin=32, hw=27, s=16, e=32)
    p = B.Plan(wl)
    assert p.num_groups == 1 and p.num_launches(True) == 1 and p.num_launches(False) == 4
    q = p.query(0)
    assert q["nlayers"] == 5
    assert q["stores_fused"] == 2 * 64 * 13 * 13                 # only the pooled tensor is written
    assert q["stores_unfused"] == 2 * (16 + 64) * 27 * 27 + 2 * 64 * 13 * 13
    assert q["mid_h"] == 2 * (q["tile_h"] - 1) + 3 + 2           # pooled tile -> 3x3/2 windows -> 3x3 conv halo
    # a padded pooling fuses as well: windows that hang over the image see -FLT_MAX there
    pp = B.Plan(W.split_fire_pool(n=1, hw=27, pp=1))
    assert pp.num_launches(True) == 1 and pp.query(0)["stores_fused"] == 64 * 14 * 14


def test_candidates_of_a_launch_can_be_listed_and_selected():
    """Paper section 3.2: the tuner searches (tile, grid) candidates; the library shows and lets a caller
    force each of them."""
    p = B.Plan(W.config(3))
    assert p.num_launches(True) == 1 and p.num_launches(False) == 3
    n = p.num_candidates(True, 0)
    assert 2 <= n <= 64
    adopted = p.candidate_info(True, 0)
    assert adopted["candidate"] == 0 and adopted["group"] == 0 and adopted["nlayers"] == 4 and adopted["is_block_kernel"] == 1
    seen = set()
    for c in range(n):
        info = p.candidate_info(True, 0, c)
        assert info["candidate"] == c and info["threads"] in (256, 512) and 0 < info["lds_bytes"] <= 160 * 1024
        assert info["workgroups"] > 0 and info["tile_h"] >= 1 and info["tile_w"] >= 1
        seen.add((info["variant"], info["threads"], info["tile_h"], info["tile_w"]))
    assert len(seen) == n          # one candidate per (kernel variant, workgroup size, tile)
    costs = [p.candidate_info(True, 0, c)["model_cost_us"] for c in range(n)]
    assert costs[0] == min(costs)
    last = p.candidate_info(True, 0, n - 1)
    p.select_candidate(True, 0, n - 1)
    now = p.candidate_info(True, 0)
    assert now["candidate"] == n - 1 and now == last
    q = p.query(0)
    assert (q["tile_h"], q["tile_w"], q["threads"], q["lds_bytes"]) == (last["tile_h"], last["tile_w"], last["threads"], last["lds_bytes"])
    # unfused launches are layers; their candidates do not touch the block's reported tiles
    u = p.candidate_info(False, 1, 0)
    assert u["group"] == -1 and u["first_layer"] == 1 and u["nlayers"] == 1
    p.select_candidate(False, 1, p.num_candidates(False, 1) - 1)
    assert p.query(0)["tile_h"] == last["tile_h"]
    for bad in ((True, 1, 0), (True, 0, n), (False, 3, 0), (True, -1, 0)):
        assert p.num_candidates(bad[0], bad[1]) == 0 or bad[2] >= p.num_candidates(bad[0], bad[1])
        with pytest.raises(B.XlError) as e:
            p.select_candidate(*bad)
        assert e.value.status == B.XL_E_GRAPH


def test_element_wise_launches_have_one_candidate():
    p = B.Plan(W.config(4))
    assert [p.num_candidates(False, l) for l in range(3)][2] == 1
    info = p.candidate_info(False, 2)
    assert info["is_block_kernel"] == 0 and info["first_layer"] == 2


def test_blocks_cut_out_of_config5_plan_like_the_network_itself():
    """The per-block GPU checks run every candidate on blocks cut out of config 5: their candidate lists must be
    the ones the whole network's plan holds."""
    full = W.config(5)
    pf = B.Plan(full)
    keys = ("variant", "tile_h", "tile_w", "threads", "cout_split", "waves_cout_1", "waves_cout_2", "chunk_channels",
            "lds_bytes", "workgroups")
    for launch in range(pf.num_launches(True)):
        gi = pf.candidate_info(True, launch)["group"]
        ps = B.Plan(W.subgraph(full, gi))
        assert ps.num_candidates(True, 0) == pf.num_candidates(True, launch)
        for c in range(ps.num_candidates(True, 0)):
            a, b = ps.candidate_info(True, 0, c), pf.candidate_info(True, launch, c)
            assert [a[k] for k in keys] == [b[k] for k in keys]


def test_shortcut_produced_after_the_first_layer_of_a_merge_block_is_rejected():
    """A fused block runs where its first layer stands; a shortcut computed by a layer listed later would be
    read before it exists."""
    with pytest.raises(B.XlError) as e:
        B.Plan(W.merge_residual_projection(shortcut_first=False))
    assert e.value.status == B.XL_E_UNSUPPORTED
    p = B.Plan(W.merge_residual_projection(shortcut_first=True))
    assert p.num_launches(True) == 2 and p.num_launches(False) == 4


def test_a_block_can_run_layer_by_layer_inside_the_fused_path():
    """The fused path launches one kernel per block, or -- for a block switched off -- the kernels of its layers
    (paper section 3.2: the tuner may only trade speed; section 3.1: reuse pays where the intermediate would
    travel off chip).  The launch list, the candidate functions and the block flags follow the switch."""
    wl = W.config(5)
    p = B.Plan(wl)
    nf, nu = p.num_launches(True), p.num_launches(False)
    assert nf == 10 and all(p.block_is_fused(g) for g in range(10))
    fire7 = next(g for g in range(p.num_groups) if "fire7" in wl.layers[wl.groups[g].layers[0]].name)
    before = [p.candidate_info(True, l) for l in range(nf)]
    p.set_block_fused(fire7, False)
    assert not p.block_is_fused(fire7)
    assert p.num_launches(True) == nf + 2            # squeeze, expand1x1, expand3x3 (the concat costs nothing)
    now = [p.candidate_info(True, l) for l in range(nf + 2)]
    pos = next(i for i, c in enumerate(before) if c["group"] == fire7)
    assert now[:pos] == before[:pos] and now[pos + 3:] == before[pos + 1:]
    layers = wl.groups[fire7].layers
    assert [c["first_layer"] for c in now[pos:pos + 3]] == [l for l in layers if wl.layers[l].op != "concat"]
    assert all(c["group"] == fire7 and c["nlayers"] == 1 for c in now[pos:pos + 3])
    # they are the unfused path's launches: selecting a candidate here selects it there
    u = next(l for l in range(nu) if p.candidate_info(False, l)["first_layer"] == layers[0])
    last = p.num_candidates(True, pos) - 1
    assert last >= 1 and p.num_candidates(False, u) == last + 1
    p.select_candidate(True, pos, last)
    assert p.candidate_info(False, u)["candidate"] == last
    assert p.query(fire7)["tile_h"] == before[pos]["tile_h"]        # the block's own report is untouched
    p.set_block_fused(fire7, True)
    assert [p.candidate_info(True, l) for l in range(nf)] == before
    one = B.Plan(W.single_conv(2, 8, 9, 9, 8, 3, pad=1))
    assert not one.block_is_fused(0)                 # a block of one layer has nothing to switch
    one.set_block_fused(0, False)
    assert one.num_launches(True) == 1
    with pytest.raises(B.XlError) as e:
        p.set_block_fused(p.num_groups, False)
    assert e.value.status == B.XL_E_GRAPH
