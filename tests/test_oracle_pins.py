"""Pins for the CPU oracle: each check fixes the oracle to something other than
itself (brute force of a differently structured definition, closed forms,
textbook special cases, a library routine in float64)."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import xlo

RNG = np.random.default_rng(20070600)


def rand(*shape):
    return RNG.standard_normal(shape).astype(np.float32)


# ---------------------------------------------------------------------------
# 1. brute force: explicit zero-padded copy + sliding windows + einsum (gather
#    form with materialised padding; the oracle is a branchy loop nest without
#    any padded copy).
# ---------------------------------------------------------------------------
def brute_conv(x, w, stride, pad, groups=1):
    x = x.astype(np.float64)
    w = w.astype(np.float64)
    n, c, h, wd = x.shape
    o, cg, kh, kw = w.shape
    xp = np.zeros((n, c, h + 2 * pad, wd + 2 * pad))
    xp[:, :, pad:pad + h, pad:pad + wd] = x
    win = np.lib.stride_tricks.sliding_window_view(xp, (kh, kw), axis=(2, 3))[:, :, ::stride, ::stride]
    og = o // groups
    outs = []
    for g in range(groups):
        outs.append(np.einsum("nchwuv,ocuv->nohw", win[:, g * cg:(g + 1) * cg], w[g * og:(g + 1) * og]))
    return np.concatenate(outs, axis=1)


@pytest.mark.parametrize("n,c,h,w,o,k,s,p,g", [
    (2, 3, 5, 5, 4, 3, 1, 1, 1),
    (1, 2, 6, 7, 3, 3, 2, 0, 1),
    (2, 4, 5, 4, 6, 1, 1, 0, 1),
    (1, 3, 7, 5, 2, 5, 1, 2, 1),
    (1, 4, 6, 6, 4, 3, 1, 1, 4),      # depthwise
    (2, 6, 5, 5, 4, 3, 2, 1, 2),
    (1, 1, 3, 3, 1, 3, 1, 1, 1),
])
def test_conv_brute_force(n, c, h, w, o, k, s, p, g):
    x = rand(n, c, h, w)
    wt = rand(o, c // g, k, k)
    got = xlo.conv2d(x, wt, s, p, g)
    ref = brute_conv(x, wt, s, p, g)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref.astype(np.float32), rtol=0, atol=0)   # double sums, one rounding


def test_conv_epilogue_order():
    """scale multiplies the bias-free sum, shift is added after, ReLU last."""
    x = rand(1, 3, 4, 4)
    wt = rand(2, 3, 3, 3)
    scale = np.array([2.0, -0.5], np.float32)
    shift = np.array([-1.0, 0.25], np.float32)
    raw = brute_conv(x, wt, 1, 1)
    ref = np.maximum(raw * scale[None, :, None, None].astype(np.float64) + shift[None, :, None, None], 0)
    got = xlo.conv2d(x, wt, 1, 1, 1, scale, shift, True)
    np.testing.assert_array_equal(got, ref.astype(np.float32))
    got_nr = xlo.conv2d(x, wt, 1, 1, 1, None, shift, False)
    np.testing.assert_array_equal(got_nr, (raw + shift[None, :, None, None]).astype(np.float32))


# ---------------------------------------------------------------------------
# 2. 1x1 convolution is a matrix product [Cout x Cin] . [Cin x HW]
# ---------------------------------------------------------------------------
def test_conv1x1_is_matmul():
    x = rand(3, 7, 5, 6)
    wt = rand(4, 7, 1, 1)
    got = xlo.conv2d(x, wt)
    ref = np.matmul(wt.reshape(4, 7).astype(np.float64), x.reshape(3, 7, 30).astype(np.float64)).reshape(3, 4, 5, 6)
    np.testing.assert_array_equal(got, ref.astype(np.float32))


# ---------------------------------------------------------------------------
# 3. delta filters pin orientation (cross-correlation) and zero padding
# ---------------------------------------------------------------------------
def test_centre_delta_is_identity():
    c = 3
    x = rand(2, c, 6, 5)
    wt = np.zeros((c, c, 3, 3), np.float32)
    for o in range(c):
        wt[o, o, 1, 1] = 1.0
    np.testing.assert_array_equal(xlo.conv2d(x, wt, 1, 1), x)


@pytest.mark.parametrize("u,v", [(0, 0), (0, 2), (2, 1), (1, 0), (2, 2)])
def test_offcentre_delta_shifts(u, v):
    """w[.., u, v] = 1 makes y[i, j] = x[i + u - 1, j + v - 1], zero where that leaves the image."""
    x = rand(1, 1, 5, 6)
    wt = np.zeros((1, 1, 3, 3), np.float32)
    wt[0, 0, u, v] = 1.0
    got = xlo.conv2d(x, wt, 1, 1)
    ref = np.zeros_like(x)
    for i in range(5):
        for j in range(6):
            ii, jj = i + u - 1, j + v - 1
            if 0 <= ii < 5 and 0 <= jj < 6:
                ref[0, 0, i, j] = x[0, 0, ii, jj]
    np.testing.assert_array_equal(got, ref)


# ---------------------------------------------------------------------------
# 4. closed forms with all-ones tensors
# ---------------------------------------------------------------------------
def _taps(n):           # in-image taps of a 3-wide window at each of n positions, pad 1
    t = np.full(n, 3.0)
    t[0] -= 1
    t[-1] -= 1
    return t


def test_all_ones_one_layer():
    cin, h, w = 5, 6, 7
    x = np.ones((1, cin, h, w), np.float32)
    wt = np.ones((2, cin, 3, 3), np.float32)
    got = xlo.conv2d(x, wt, 1, 1)
    ref = cin * np.outer(_taps(h), _taps(w))
    assert got[0, 0, 0, 0] == 4 * cin and got[0, 0, 0, 3] == 6 * cin and got[0, 0, 2, 3] == 9 * cin
    np.testing.assert_array_equal(got[0, 0], ref.astype(np.float32))
    np.testing.assert_array_equal(got[0, 1], ref.astype(np.float32))


def test_all_ones_two_stacked_layers_prezeroed_intermediate():
    """Second layer sees ZERO outside the image, not layer 1 evaluated there:
    out = C1*Cin * (sum of row taps over the in-image window) x (same for columns)."""
    cin, c1, h, w = 3, 4, 6, 5
    x = np.ones((1, cin, h, w), np.float32)
    w1 = np.ones((c1, cin, 3, 3), np.float32)
    w2 = np.ones((2, c1, 3, 3), np.float32)
    mid = xlo.conv2d(x, w1, 1, 1, 1, None, np.ones(c1, np.float32), True)        # bias +1: a wrong border shows
    got = xlo.conv2d(mid, w2, 1, 1)

    def win_sum(t):     # sum of t over the in-image 3-window at each position
        p = np.concatenate([[0.0], t, [0.0]])
        return p[:-2] + p[1:-1] + p[2:]
    rows, cols = _taps(h), _taps(w)
    # mid = cin*rows x cols + 1  ->  sum over window = cin * S(rows) x S(cols) + (#taps rows) x (#taps cols)
    ref = c1 * (cin * np.outer(win_sum(rows), win_sum(cols)) + np.outer(_taps(h), _taps(w)))
    np.testing.assert_array_equal(got[0, 0], ref.astype(np.float32))


# ---------------------------------------------------------------------------
# 5. invariants
# ---------------------------------------------------------------------------
def test_linearity():
    x1, x2 = rand(1, 4, 6, 6), rand(1, 4, 6, 6)
    wt = rand(3, 4, 3, 3)
    lhs = xlo.conv2d(2.0 * x1 - 3.0 * x2, wt, 1, 1).astype(np.float64)
    rhs = 2.0 * xlo.conv2d(x1, wt, 1, 1).astype(np.float64) - 3.0 * xlo.conv2d(x2, wt, 1, 1)
    np.testing.assert_allclose(lhs, rhs, rtol=0, atol=2e-5)


def test_batch_independence():
    x = rand(3, 4, 5, 5)
    wt = rand(2, 4, 3, 3)
    full = xlo.conv2d(x, wt, 1, 1)
    for n in range(3):
        np.testing.assert_array_equal(full[n:n + 1], xlo.conv2d(x[n:n + 1], wt, 1, 1))


def test_concat_is_two_independent_convs():
    x = rand(2, 4, 5, 5)
    wa, wb = rand(3, 4, 1, 1), rand(2, 4, 3, 3)
    a, b = xlo.conv2d(x, wa), xlo.conv2d(x, wb, 1, 1)
    y = xlo.concat_channels(a, b)
    np.testing.assert_array_equal(y[:, :3], a)
    np.testing.assert_array_equal(y[:, 3:], b)
    np.testing.assert_array_equal(y, np.concatenate([a, b], axis=1))


def test_maxpool_pad_equivalence_on_nonnegative_input():
    """Ignoring out-of-image taps equals zero padding when the input is post-ReLU."""
    x = np.maximum(rand(2, 3, 7, 7), 0)
    got = xlo.maxpool2d(x, 3, 2, 1)
    xp = np.zeros((2, 3, 9, 9), np.float32)
    xp[:, :, 1:8, 1:8] = x
    win = np.lib.stride_tricks.sliding_window_view(xp, (3, 3), axis=(2, 3))[:, :, ::2, ::2]
    np.testing.assert_array_equal(got, win.max(axis=(4, 5)))


def test_maxpool_ignores_padding_on_negative_input():
    x = -np.abs(rand(1, 1, 4, 4)) - 1.0
    got = xlo.maxpool2d(x, 3, 2, 1)
    assert got.max() < 0            # a zero pad would have produced 0 at the border
    assert got[0, 0, 0, 0] == x[0, 0, 0:2, 0:2].max()


def test_global_avgpool_and_add():
    x = np.full((2, 3, 13, 13), 0.3, np.float32)
    np.testing.assert_allclose(xlo.global_avgpool(x), np.float32(0.3), rtol=1e-7)
    y = rand(2, 3, 4, 5)
    np.testing.assert_allclose(xlo.global_avgpool(y)[:, :, 0, 0], y.astype(np.float64).mean(axis=(2, 3)), rtol=1e-6, atol=1e-7)
    a, b = rand(5, 7), rand(5, 7)
    np.testing.assert_array_equal(xlo.add(a, b), a + b)
    np.testing.assert_array_equal(xlo.add(a, b, True), np.maximum(a + b, 0))


# ---------------------------------------------------------------------------
# 7. library cross-check in float64 (torch CPU), random shapes
# ---------------------------------------------------------------------------
@pytest.mark.parametrize("seed", range(6))
def test_against_torch_float64(seed):
    r = np.random.default_rng(seed)
    n, g = int(r.integers(1, 3)), int(r.choice([1, 1, 2]))
    c, o = g * int(r.integers(1, 5)), g * int(r.integers(1, 5))
    k, s = int(r.choice([1, 3, 5])), int(r.choice([1, 2]))
    p = int(r.integers(0, k // 2 + 1))
    h, w = int(r.integers(k, 12)), int(r.integers(k, 12))
    x = r.standard_normal((n, c, h, w)).astype(np.float32)
    wt = r.standard_normal((o, c // g, k, k)).astype(np.float32)
    b = r.standard_normal(o).astype(np.float32)
    ref = F.conv2d(torch.from_numpy(x).double(), torch.from_numpy(wt).double(), torch.from_numpy(b).double(),
                   stride=s, padding=p, groups=g).numpy()
    got = xlo.conv2d(x, wt, s, p, g, None, b, False)
    np.testing.assert_allclose(got, ref, rtol=1e-6, atol=1e-6)
    if h >= 3 and w >= 3:
        pk, ps, pp = 3, int(r.choice([1, 2])), int(r.choice([0, 1]))
        refp = F.max_pool2d(torch.from_numpy(x), pk, ps, pp).numpy()
        np.testing.assert_array_equal(xlo.maxpool2d(x, pk, ps, pp), refp)


def test_bad_sizes_rejected():
    with pytest.raises(ValueError):
        xlo.conv2d(rand(1, 3, 2, 2), rand(2, 3, 5, 5))           # window larger than padded image
    with pytest.raises(ValueError):
        xlo.conv2d(rand(1, 3, 4, 4), rand(2, 2, 3, 3))           # channel mismatch
    with pytest.raises(ValueError):
        xlo.add(rand(2, 3), rand(3, 2))
