"""GPU parity on seeded random block shapes: every block kind, odd extents and channel counts, both
arithmetic modes, planner's choice and tuned plan.  Same bar as everywhere: |g - o| <= 1e-4 + 1e-4 |o|."""
import random

import pytest

import xl_workloads as W
from test_gpu_parity import run_both

pytestmark = pytest.mark.gpu


def random_workload(rng):
    kind = rng.choice(["straight", "pool", "fire", "firepool", "merge", "gap", "depthwise", "two_producers", "five"])
    n, h, w = rng.choice([1, 2, 3]), rng.randint(5, 40), rng.randint(5, 40)
    cin = rng.choice([3, 8, 13, 16, 24, 40, 64, 72])
    c1 = rng.choice([8, 16, 20, 32, 48, 64])
    c2 = rng.choice([8, 16, 24, 32, 64, 100])
    k1, k2 = rng.choice([1, 3]), rng.choice([1, 3])
    if kind == "straight":
        return W.straight_generic(n, cin, h, w, c1, k1, k1 // 2, rng.choice([1, 1, 2]), c2, k2, k2 // 2, 1,
                                  bn1=rng.random() < .5, bn2=rng.random() < .5)
    if kind == "five":
        return W.straight_generic(n, cin, h, w, c1, k1, k1 // 2, 1, c2, 5, 2, 1)
    if kind == "pool":
        return W.conv_pool_generic(n, cin, h, w, c1, k1, k1 // 2, rng.choice([1, 2]), 3, 2, rng.choice([0, 1]),
                                   bn=rng.random() < .5)
    if kind == "fire":
        return W.config(3, n=n, hw=h, cin=cin, s=rng.choice([8, 16, 48]), e=rng.choice([16, 64, 96]))
    if kind == "firepool":
        return W.split_fire_pool(n=n, cin=cin, hw=max(h, 7), s=rng.choice([8, 16, 48]), e=rng.choice([16, 32, 96]),
                                 pk=rng.choice([2, 3]), ps=2, pp=rng.choice([0, 0, 1]))
    if kind == "merge":
        return W.config(4, n=n, hw=h, c=rng.choice([16, 32, 64]))
    if kind == "gap":
        return W.conv_gap_generic(n, cin, min(h, 14), min(w, 14), c2, k1, k1 // 2, 1)
    if kind == "depthwise":
        return W.depthwise_pointwise(n, rng.choice([6, 16, 24]), h, w, c2)
    return W.merge_two_producers(n, c=rng.choice([16, 24, 64]), h=h, w=w, cmid=rng.choice([32, 40, 128]),
                                 cout=rng.choice([16, 20, 64]))


@pytest.mark.parametrize("seed", range(24))
def test_random_block(seed):
    wl = random_workload(random.Random(7000 + seed))
    run_both(wl)
    run_both(wl, precision=1)
    run_both(wl, tune=True, precision=seed % 2)
