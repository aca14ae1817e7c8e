"""Pins for the fp64 direct-sum oracle (CPU only).

The paper prints no numeric worked example, so the oracle is tied to things
that are fixed independently of it: hand-worked values (tests/golden), closed
forms for degenerate inputs, algebraic invariants of Eqs. (1)-(3), library
routines that the passes reduce to for a single map pair, and an independent
pure-Python loop nest on tiny shapes.
"""
import itertools
import json
import os

import numpy as np
import pytest
import scipy.signal as sps
import torch

from oracle import direct

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rng(seed):
    return np.random.Generator(np.random.Philox(key=seed))


def rand_layer(seed, S, f, fo, n, k):
    r = rng(seed)
    no = n - k + 1
    return (r.uniform(-1, 1, (S, f, n, n)), r.standard_normal((fo, f, k, k)),
            r.standard_normal((S, fo, no, no)))


# ---------------------------------------------------------------- hand cases

def test_hand_case_3x3_golden():
    gold = json.load(open(os.path.join(GOLD, "hand_case_3x3.json")))
    x = np.array(gold["x"], float).reshape(1, 1, 3, 3)
    w = np.array(gold["w"], float).reshape(1, 1, 2, 2)
    g = np.array(gold["g"], float).reshape(1, 1, 2, 2)
    assert np.array_equal(direct.fprop(x, w)[0, 0], np.array(gold["fprop_y"], float))
    assert not np.array_equal(direct.fprop(x, w)[0, 0], np.array(gold["true_convolution_y_would_be"], float))
    assert np.array_equal(direct.bprop(g, w, 3)[0, 0], np.array(gold["bprop_dx"], float))
    assert np.array_equal(direct.accgrad(g, x, 2)[0, 0], np.array(gold["accgrad_dw"], float))


def test_two_input_maps_by_hand():
    # y = x0 (star) w0 + x1 (star) w1 with 1x2 effective taps; numbers small enough to do on paper.
    x = np.zeros((1, 2, 2, 2)); x[0, 0] = [[1, 2], [3, 4]]; x[0, 1] = [[10, 20], [30, 40]]
    w = np.zeros((1, 2, 2, 2)); w[0, 0] = [[1, 0], [0, 0]]; w[0, 1] = [[0, 0], [0, 2]]
    # single output pixel: 1*x0[0,0] + 2*x1[1,1] = 1 + 80
    assert direct.fprop(x, w).tolist() == [[[[81.0]]]]


@pytest.mark.parametrize("a0,b0", [(0, 0), (0, 2), (2, 0), (1, 2), (2, 2)])
def test_delta_kernel_selects_shifted_window(a0, b0):
    # w = delta at (a0,b0): y = x[a0:a0+no, b0:b0+no] -- pins orientation (no flip) and crop offset.
    S, f, fo, n, k = 2, 3, 2, 7, 3
    x, _, _ = rand_layer(1, S, f, fo, n, k)
    w = np.zeros((fo, f, k, k)); w[1, 2, a0, b0] = 1.0
    y = direct.fprop(x, w)
    no = n - k + 1
    assert np.array_equal(y[:, 1], x[:, 2, a0:a0 + no, b0:b0 + no])
    assert np.all(y[:, 0] == 0)


@pytest.mark.parametrize("a0,b0", [(0, 0), (0, 2), (2, 1)])
def test_delta_kernel_bprop_places_gradient(a0, b0):
    # adjoint of a shifted-window read is a shifted write: dx[:, i, a0:a0+no, b0:b0+no] = g[:, j]
    S, f, fo, n, k = 2, 3, 2, 6, 3
    _, _, g = rand_layer(2, S, f, fo, n, k)
    w = np.zeros((fo, f, k, k)); w[1, 0, a0, b0] = 1.0
    dx = direct.bprop(g, w, n)
    no = n - k + 1
    exp = np.zeros((S, f, n, n)); exp[:, 0, a0:a0 + no, b0:b0 + no] = g[:, 1]
    assert np.array_equal(dx, exp)


def test_delta_gradient_accgrad_reads_window():
    # g = delta at (s0,j0,p0,q0): dw[j0,i,a,b] = x[s0,i,p0+a,q0+b]
    S, f, fo, n, k = 3, 2, 2, 6, 3
    x, _, _ = rand_layer(3, S, f, fo, n, k)
    no = n - k + 1
    g = np.zeros((S, fo, no, no)); g[2, 1, 1, 3] = 1.0
    dw = direct.accgrad(g, x, k)
    assert np.array_equal(dw[1], x[2, :, 1:1 + k, 3:3 + k])
    assert np.all(dw[0] == 0)


def test_k1_is_a_channel_mixing_matrix():
    S, f, fo, n = 2, 4, 3, 5
    x, w, g = rand_layer(4, S, f, fo, n, 1)
    y = direct.fprop(x, w)
    np.testing.assert_allclose(y, np.einsum("ji,sipq->sjpq", w[:, :, 0, 0], x), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(direct.bprop(g, w, n), np.einsum("ji,sjpq->sipq", w[:, :, 0, 0], g), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(direct.accgrad(g, x, 1)[:, :, 0, 0], np.einsum("sjpq,sipq->ji", g, x), rtol=1e-13, atol=1e-13)


def test_k_equals_n_is_a_full_dot_product():
    S, f, fo, n = 2, 3, 2, 4
    x, w, g = rand_layer(5, S, f, fo, n, n)
    y = direct.fprop(x, w)
    assert y.shape == (S, fo, 1, 1)
    np.testing.assert_allclose(y[:, :, 0, 0], np.einsum("siab,jiab->sj", x, w), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(direct.bprop(g, w, n), np.einsum("sj,jiab->siab", g[:, :, 0, 0], w), rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(direct.accgrad(g, x, n), np.einsum("sj,siab->jiab", g[:, :, 0, 0], x), rtol=1e-13, atol=1e-13)


def test_all_ones_closed_forms():
    S, f, fo, n, k = 2, 3, 4, 9, 4
    no = n - k + 1
    x = np.ones((S, f, n, n)); w = np.ones((fo, f, k, k)); g = np.ones((S, fo, no, no))
    assert np.all(direct.fprop(x, w) == f * k * k)
    assert np.all(direct.accgrad(g, x, k) == S * no * no)
    taps = np.array([min(p + 1, k, n - p, no) for p in range(n)], float)
    exp = fo * np.outer(taps, taps)
    assert np.array_equal(direct.bprop(g, w, n), np.broadcast_to(exp, (S, f, n, n)))


# ---------------------------------------------------------------- invariants

def test_linearity_in_each_argument():
    S, f, fo, n, k = 2, 3, 2, 8, 3
    x1, w1, g1 = rand_layer(6, S, f, fo, n, k)
    x2, w2, g2 = rand_layer(7, S, f, fo, n, k)
    a, b = 0.75, -1.5
    for fn, lhs, rhs in (
        (lambda x: direct.fprop(x, w1), a * x1 + b * x2, (x1, x2)),
        (lambda w: direct.fprop(x1, w), a * w1 + b * w2, (w1, w2)),
        (lambda g: direct.bprop(g, w1, n), a * g1 + b * g2, (g1, g2)),
        (lambda w: direct.bprop(g1, w, n), a * w1 + b * w2, (w1, w2)),
        (lambda g: direct.accgrad(g, x1, k), a * g1 + b * g2, (g1, g2)),
        (lambda x: direct.accgrad(g1, x, k), a * x1 + b * x2, (x1, x2)),
    ):
        np.testing.assert_allclose(fn(lhs), a * fn(rhs[0]) + b * fn(rhs[1]), rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("dims", [(3, 4, 5, 9, 3), (2, 1, 3, 6, 6), (2, 5, 2, 7, 1), (1, 3, 3, 8, 5)])
def test_adjoint_identity(dims):
    # <fprop(x,w), g> = <x, bprop(g,w)> = <w, accGrad(g,x)>
    S, f, fo, n, k = dims
    x, w, g = rand_layer(8, *dims)
    a = np.vdot(direct.fprop(x, w), g)
    b = np.vdot(x, direct.bprop(g, w, n))
    c = np.vdot(w, direct.accgrad(g, x, k))
    assert abs(a - b) <= 1e-12 * abs(a) and abs(a - c) <= 1e-12 * abs(a)


def test_permutation_equivariance():
    S, f, fo, n, k = 3, 4, 5, 7, 3
    x, w, g = rand_layer(9, S, f, fo, n, k)
    r = rng(10)
    ps, pf, pfo = r.permutation(S), r.permutation(f), r.permutation(fo)
    y = direct.fprop(x, w)
    np.testing.assert_allclose(direct.fprop(x[ps][:, pf], w[pfo][:, pf]), y[ps][:, pfo], rtol=1e-12, atol=1e-13)
    dx = direct.bprop(g, w, n)
    np.testing.assert_allclose(direct.bprop(g[ps][:, pfo], w[pfo][:, pf], n), dx[ps][:, pf], rtol=1e-12, atol=1e-13)
    dw = direct.accgrad(g, x, k)
    np.testing.assert_allclose(direct.accgrad(g[ps][:, pfo], x[ps][:, pf], k), dw[pfo][:, pf], rtol=1e-12, atol=1e-13)


def test_translation_of_input_shifts_interior_of_output():
    S, f, fo, n, k = 1, 2, 2, 10, 3
    x, w, _ = rand_layer(11, S, f, fo, n, k)
    y = direct.fprop(x, w)
    xs = np.zeros_like(x); xs[:, :, 1:, 2:] = x[:, :, :-1, :-2]
    ys = direct.fprop(xs, w)
    np.testing.assert_allclose(ys[:, :, 1:, 2:], y[:, :, :-1, :-2], rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- library special cases

@pytest.mark.parametrize("n,k", [(8, 3), (9, 4), (6, 6), (7, 1)])
def test_single_map_pair_matches_scipy(n, k):
    x, w, g = rand_layer(12, 1, 1, 1, n, k)
    np.testing.assert_allclose(direct.fprop(x, w)[0, 0], sps.correlate2d(x[0, 0], w[0, 0], "valid"), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(direct.bprop(g, w, n)[0, 0], sps.convolve2d(g[0, 0], w[0, 0], "full"), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(direct.accgrad(g, x, k)[0, 0], sps.correlate2d(x[0, 0], g[0, 0], "valid"), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("dims", [(3, 4, 5, 12, 5), (2, 3, 2, 16, 3), (2, 2, 3, 9, 9)])
def test_whole_layer_matches_torch_conv2d_and_autograd(dims):
    S, f, fo, n, k = dims
    x, w, g = rand_layer(13, *dims)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt)
    yt.backward(torch.tensor(g, dtype=torch.float64))
    np.testing.assert_allclose(direct.fprop(x, w), yt.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(direct.bprop(g, w, n), xt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(direct.accgrad(g, x, k), wt.grad.numpy(), rtol=1e-11, atol=1e-12)


# ---------------------------------------------------------------- brute force on tiny inputs

def brute(x, w, g):
    S, f, n, _ = x.shape
    fo, _, k, _ = w.shape
    no = n - k + 1
    y = np.zeros((S, fo, no, no)); dx = np.zeros_like(x); dw = np.zeros_like(w)
    for s, j, i, p, q, a, b in itertools.product(range(S), range(fo), range(f), range(no), range(no), range(k), range(k)):
        y[s, j, p, q] += x[s, i, p + a, q + b] * w[j, i, a, b]
        dx[s, i, p + a, q + b] += g[s, j, p, q] * w[j, i, a, b]
        dw[j, i, a, b] += g[s, j, p, q] * x[s, i, p + a, q + b]
    return y, dx, dw


@pytest.mark.parametrize("dims", [(2, 3, 2, 3, 2), (3, 2, 3, 3, 3), (1, 1, 1, 3, 1), (2, 2, 3, 3, 2)])
def test_brute_force_tiny(dims):
    x, w, g = rand_layer(14, *dims)
    y, dx, dw = brute(x, w, g)
    np.testing.assert_allclose(direct.fprop(x, w), y, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(direct.bprop(g, w, dims[3]), dx, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(direct.accgrad(g, x, dims[4]), dw, rtol=1e-13, atol=1e-13)


# ---------------------------------------------------------------- restricted-unit interface

def test_unit_subsets_equal_slices_of_the_full_result():
    S, f, fo, n, k = 3, 4, 5, 8, 3
    x, w, g = rand_layer(15, S, f, fo, n, k)
    y, dx, dw = direct.fprop(x, w), direct.bprop(g, w, n), direct.accgrad(g, x, k)
    u = np.array([14, 0, 7, 3])
    assert np.array_equal(direct.fprop(x, w, u), y.reshape(S * fo, *y.shape[2:])[u])
    u = np.array([11, 2, 5])
    assert np.array_equal(direct.bprop(g, w, n, u), dx.reshape(S * f, n, n)[u])
    u = np.array([19, 4, 0])
    assert np.array_equal(direct.accgrad(g, x, k, u), dw.reshape(fo * f, k, k)[u])


def test_results_do_not_depend_on_thread_schedule():
    x, w, g = rand_layer(16, 4, 3, 5, 10, 3)
    assert np.array_equal(direct.fprop(x, w), direct.fprop(x, w))
    assert np.array_equal(direct.accgrad(g, x, 3), direct.accgrad(g, x, 3))


def test_shape_errors():
    with pytest.raises(ValueError):
        direct.fprop(np.zeros((1, 2, 4, 4)), np.zeros((1, 3, 2, 2)))
    with pytest.raises(ValueError):
        direct.fprop(np.zeros((1, 2, 4, 4)), np.zeros((1, 2, 5, 5)))
    with pytest.raises(ValueError):
        direct.bprop(np.zeros((1, 2, 3, 3)), np.zeros((2, 2, 2, 2)), 5)


# ---------------------------------------------------------------- rectangular maps and kernels
# (Sec. 2.1 writes square maps only to keep the notation short; a wrong axis, a transposed
# kernel or swapped height / width in any of the three loops fails at least one of these.)

def rand_rect(seed, S, f, fo, nh, nw, kh, kw):
    r = rng(seed)
    return (r.uniform(-1, 1, (S, f, nh, nw)), r.standard_normal((fo, f, kh, kw)),
            r.standard_normal((S, fo, nh - kh + 1, nw - kw + 1)))


RECT = [(2, 3, 2, 7, 11, 3, 2), (1, 2, 3, 12, 5, 1, 4), (2, 2, 2, 6, 9, 6, 2), (3, 1, 2, 5, 8, 2, 8)]


@pytest.mark.parametrize("dims", RECT)
def test_rectangular_single_pairs_match_scipy(dims):
    S, f, fo, nh, nw, kh, kw = dims
    x, w, g = rand_rect(21, 1, 1, 1, nh, nw, kh, kw)
    np.testing.assert_allclose(direct.fprop(x, w)[0, 0], sps.correlate2d(x[0, 0], w[0, 0], "valid"), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(direct.bprop(g, w, (nh, nw))[0, 0], sps.convolve2d(g[0, 0], w[0, 0], "full"), rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(direct.accgrad(g, x, (kh, kw))[0, 0], sps.correlate2d(x[0, 0], g[0, 0], "valid"), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("dims", RECT)
def test_rectangular_layer_matches_torch_and_adjoint_identity(dims):
    S, f, fo, nh, nw, kh, kw = dims
    x, w, g = rand_rect(22, *dims)
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wt = torch.tensor(w, dtype=torch.float64, requires_grad=True)
    yt = torch.nn.functional.conv2d(xt, wt)
    yt.backward(torch.tensor(g, dtype=torch.float64))
    y, dx, dw = direct.fprop(x, w), direct.bprop(g, w, (nh, nw)), direct.accgrad(g, x, (kh, kw))
    assert y.shape == g.shape and dx.shape == x.shape and dw.shape == w.shape
    np.testing.assert_allclose(y, yt.detach().numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(dw, wt.grad.numpy(), rtol=1e-11, atol=1e-12)
    a, b, c = np.vdot(y, g), np.vdot(x, dx), np.vdot(w, dw)
    assert abs(a - b) <= 1e-12 * abs(a) + 1e-12 and abs(a - c) <= 1e-12 * abs(a) + 1e-12


def test_rectangular_brute_force_and_delta_kernel():
    S, f, fo, nh, nw, kh, kw = 2, 2, 2, 4, 3, 2, 3
    x, w, g = rand_rect(23, S, f, fo, nh, nw, kh, kw)
    noh, now = nh - kh + 1, nw - kw + 1
    y = np.zeros((S, fo, noh, now)); dx = np.zeros_like(x); dw = np.zeros_like(w)
    for s, j, i, p, q, a, b in itertools.product(range(S), range(fo), range(f), range(noh), range(now), range(kh), range(kw)):
        y[s, j, p, q] += x[s, i, p + a, q + b] * w[j, i, a, b]
        dx[s, i, p + a, q + b] += g[s, j, p, q] * w[j, i, a, b]
        dw[j, i, a, b] += g[s, j, p, q] * x[s, i, p + a, q + b]
    np.testing.assert_allclose(direct.fprop(x, w), y, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(direct.bprop(g, w, (nh, nw)), dx, rtol=1e-13, atol=1e-13)
    np.testing.assert_allclose(direct.accgrad(g, x, (kh, kw)), dw, rtol=1e-13, atol=1e-13)
    # delta kernel at (a0, b0) of a 2 x 4 kernel selects the window shifted by (a0, b0)
    x = rng(24).uniform(-1, 1, (1, 1, 6, 9))
    for a0, b0 in ((0, 0), (1, 3), (0, 2)):
        wd = np.zeros((1, 1, 2, 4)); wd[0, 0, a0, b0] = 1.0
        assert np.array_equal(direct.fprop(x, wd)[0, 0], x[0, 0, a0:a0 + 5, b0:b0 + 6])


# ---------------------------------------------------------------- true-convolution reading of "*"

@pytest.mark.parametrize("dims", [(1, 1, 1, 8, 8, 3, 3), (2, 3, 2, 7, 11, 3, 2), (2, 2, 3, 9, 6, 4, 5)])
def test_true_convolution_option(dims):
    """With true_conv the passes are the valid true convolution (scipy convolve2d) and its adjoints."""
    S, f, fo, nh, nw, kh, kw = dims
    x, w, g = rand_rect(31, *dims)
    y = direct.fprop(x, w, true_conv=True)
    ref = np.zeros_like(y)
    for s, j, i in itertools.product(range(S), range(fo), range(f)):
        ref[s, j] += sps.convolve2d(x[s, i], w[j, i], "valid")
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-12)
    dx = direct.bprop(g, w, (nh, nw), true_conv=True)
    dw = direct.accgrad(g, x, (kh, kw), true_conv=True)
    a, b, c = np.vdot(y, g), np.vdot(x, dx), np.vdot(w, dw)
    assert abs(a - b) <= 1e-12 * abs(a) + 1e-12 and abs(a - c) <= 1e-12 * abs(a) + 1e-12
    # gradient by finite differences of <fprop(x, w), g> in one kernel entry (linear in w: exact up to rounding)
    e = np.zeros_like(w); e[fo - 1, 0, kh - 1, 0] = 1.0
    fd = np.vdot(direct.fprop(x, w + e, true_conv=True) - y, g)
    assert abs(fd - dw[fo - 1, 0, kh - 1, 0]) <= 1e-10 * (1 + abs(fd))
    # and it differs from the cross-correlation unless the kernel is symmetric
    assert not np.allclose(y, direct.fprop(x, w))
