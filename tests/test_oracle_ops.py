"""Pins for the oracle's single operations (no GPU): each is checked against something
other than itself -- a library routine, a closed form, a special case or brute force."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from oracle import ops

A, B = 1.7159, 0.6666


def _rand_table(rng, mo, mi, p=0.5):
    t = (rng.random((mo, mi)) < p).astype(np.uint8)
    for j in range(mo):
        if not t[j].any():
            t[j, rng.integers(mi)] = 1
    return t


def _dense_from_csr(w_csr, table, k_y, k_x):
    """Scatter the oracle's per-connection kernel list into a dense [mo, mi, ky, kx] array
    (absent connections stay zero).  Index work only."""
    mo, mi = table.shape
    dense = np.zeros((mo, mi, k_y, k_x))
    slot = 0
    for j in range(mo):
        for i in range(mi):
            if table[j, i]:
                dense[j, i] = w_csr[slot]
                slot += 1
    assert slot == w_csr.shape[0]
    return dense


# ------------------------------------------------------------------ activation

def test_activation_constants_and_closed_forms():
    # Sec. 4: y(a) = 1.7159 tanh(0.6666 a)
    for a in (-3.0, -0.5, 0.0, 0.1, 2.0):
        assert ops.act(a) == pytest.approx(A * np.tanh(B * a), rel=1e-15, abs=1e-300)
    assert ops.act(0.0) == 0.0
    assert ops.act(50.0) == pytest.approx(A, rel=1e-12)            # saturates at the scale factor
    assert ops.act(-1.3) == -ops.act(1.3)                           # odd function
    # slope at the origin is A*B; derivative from the output matches a central difference
    assert ops.act_deriv_from_output(0.0) == pytest.approx(A * B, rel=1e-15)
    for a in (-1.2, -0.1, 0.3, 1.7):
        h = 1e-6
        fd = (ops.act(a + h) - ops.act(a - h)) / (2 * h)
        assert ops.act_deriv_from_output(ops.act(a)) == pytest.approx(fd, rel=1e-8)


# ------------------------------------------------------------------ convolution forward

@pytest.mark.parametrize("mi,mo,h,w,k,s,sparse", [
    (1, 3, 9, 9, 4, 0, False), (3, 5, 11, 13, 5, 0, False), (4, 6, 12, 12, 5, 1, False),
    (4, 6, 13, 10, 3, 2, False), (6, 7, 10, 10, 3, 0, True), (5, 4, 12, 11, 2, 1, True),
    (2, 3, 7, 7, 1, 0, False), (2, 3, 8, 8, 1, 2, True),
])
def test_conv_forward_vs_library_conv2d(mi, mo, h, w, k, s, sparse):
    """S = 0 and a full table is a library conv2d (correlation, no flip); S > 0 is conv2d
    with stride S + 1; a sparse table is the full layer with absent kernels set to zero."""
    rng = np.random.default_rng(100 + mi * 7 + mo + k + s)
    x = rng.standard_normal((mi, h, w))
    table = _rand_table(rng, mo, mi) if sparse else np.ones((mo, mi), dtype=np.uint8)
    wk = rng.standard_normal((int(table.sum()), k, k)) * 0.3
    b = rng.standard_normal(mo) * 0.1
    got = ops.conv_forward(x, b, wk, mo, k, k, s, s, table=table if sparse else None, apply_act=False)
    dense = _dense_from_csr(wk, table, k, k)
    want = torch.nn.functional.conv2d(torch.from_numpy(x)[None], torch.from_numpy(dense),
                                      torch.from_numpy(b), stride=s + 1)[0].numpy()
    assert got.shape == want.shape
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)
    got_act = ops.conv_forward(x, b, wk, mo, k, k, s, s, table=table if sparse else None)
    np.testing.assert_allclose(got_act, A * np.tanh(B * want), rtol=1e-12, atol=1e-12)


def test_conv_rectangular_kernel_and_unequal_skips():
    """Sec. 2.2 allows Kx != Ky and Sx != Sy."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 12, 15))
    wk = rng.standard_normal((6, 3, 4))          # ky = 3, kx = 4
    b = rng.standard_normal(3)
    got = ops.conv_forward(x, b, wk, 3, 3, 4, 1, 2, apply_act=False)
    want = torch.nn.functional.conv2d(torch.from_numpy(x)[None],
                                      torch.from_numpy(wk.reshape(3, 2, 3, 4)),
                                      torch.from_numpy(b), stride=(2, 3))[0].numpy()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_conv_kernel_as_large_as_input_is_a_fully_connected_layer():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((3, 5, 5))
    wk = rng.standard_normal((4 * 3, 5, 5))
    b = rng.standard_normal(4)
    got = ops.conv_forward(x, b, wk, 4, 5, 5, apply_act=False)
    want = wk.reshape(4, 75) @ x.ravel() + b
    np.testing.assert_allclose(got.ravel(), want, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(ops.fc_forward(x, b, wk.reshape(4, 75)), want, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("s", [0, 1, 2])
def test_conv_single_unit_tap_is_a_shifted_subsampled_copy(s):
    """One tap equal to 1 at (a, b), everything else 0: out[y, x] = in[y(S+1)+a, x(S+1)+b]."""
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 11, 12))
    k = 3
    for a, b in itertools.product(range(k), range(k)):
        wk = np.zeros((2, k, k))
        wk[1, a, b] = 1.0                          # output map 0 reads input map 1 only
        got = ops.conv_forward(x, np.zeros(1), wk, 1, k, k, s, s, apply_act=False)[0]
        ho, wo = got.shape
        want = x[1, a:a + (ho - 1) * (s + 1) + 1:s + 1, b:b + (wo - 1) * (s + 1) + 1:s + 1]
        np.testing.assert_array_equal(got, want)


def test_conv_bias_only():
    x = np.zeros((2, 6, 6))
    wk = np.ones((6, 3, 3))
    b = np.array([0.3, -0.2, 1.0])
    got = ops.conv_forward(x, b, wk, 3, 3, 3)
    for j in range(3):
        np.testing.assert_allclose(got[j], A * np.tanh(B * b[j]), rtol=1e-15)


# ------------------------------------------------------------------ max-pooling

@pytest.mark.parametrize("m,h,w,ky,kx", [(3, 6, 6, 2, 2), (2, 9, 9, 3, 3), (2, 8, 12, 4, 4),
                                         (1, 6, 9, 2, 3), (2, 5, 5, 1, 1)])
def test_maxpool_brute_force(m, h, w, ky, kx):
    rng = np.random.default_rng(11)
    x = rng.standard_normal((m, h, w))
    out, arg = ops.maxpool_forward(x, ky, kx)
    for j, y, xx in itertools.product(range(m), range(h // ky), range(w // kx)):
        win = x[j, y * ky:(y + 1) * ky, xx * kx:(xx + 1) * kx]
        assert out[j, y, xx] == win.max()
        assert arg[j, y, xx] == int(np.argmax(win.ravel()))   # numpy: first maximum, row-major


def test_maxpool_ties_take_the_first_in_row_major_order():
    x = np.full((2, 4, 6), 0.25)
    out, arg = ops.maxpool_forward(x, 2, 3)
    assert (arg == 0).all() and (out == 0.25).all()
    x = np.zeros((1, 2, 2))
    x[0, 0, 1] = x[0, 1, 0] = 1.0
    _, arg = ops.maxpool_forward(x, 2, 2)
    assert arg[0, 0, 0] == 1


def test_maxpool_k1_is_identity():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((2, 4, 5))
    out, arg = ops.maxpool_forward(x, 1, 1)
    np.testing.assert_array_equal(out, x)
    assert (arg == 0).all()


def test_maxpool_rejects_non_dividing_rectangle():
    with pytest.raises(oracle.binding.OracleError):
        ops.maxpool_forward(np.zeros((1, 5, 6)), 2, 2)


def test_maxpool_backward_routes_to_the_winner_only():
    rng = np.random.default_rng(13)
    x = rng.standard_normal((3, 6, 8))
    out, arg = ops.maxpool_forward(x, 2, 2)
    g = rng.standard_normal(out.shape)
    gi = ops.maxpool_backward(g, arg, 6, 8, 2, 2)
    # one non-zero per window, at the maximum, carrying the window's gradient
    for j, y, xx in itertools.product(range(3), range(3), range(4)):
        win = gi[j, 2 * y:2 * y + 2, 2 * xx:2 * xx + 2]
        assert np.count_nonzero(win) == 1
        dy, dx = np.unravel_index(np.argmax(x[j, 2 * y:2 * y + 2, 2 * xx:2 * xx + 2]), (2, 2))
        assert win[dy, dx] == g[j, y, xx]
    assert gi.sum() == pytest.approx(g.sum(), rel=1e-13)
    # library witness
    xt = torch.from_numpy(x)[None].requires_grad_(True)
    torch.nn.functional.max_pool2d(xt, 2).backward(torch.from_numpy(g)[None])
    np.testing.assert_array_equal(gi, xt.grad[0].numpy())


# ------------------------------------------------------------------ deltas through a conv layer

CASES = [(mi, mo, h, w, k, s, sp)
         for (mi, mo) in [(1, 2), (3, 4)]
         for (h, w) in [(7, 7), (9, 8), (12, 11)]
         for k in [1, 2, 3, 4, 5]
         for s in [0, 1, 2]
         for sp in [False, True]
         if h >= k and w >= k]


@pytest.mark.parametrize("mi,mo,h,w,k,s,sparse", CASES)
def test_pull_equals_push(mi, mo, h, w, k, s, sparse):
    """The index inequalities of Sec. 3.3 (pull) against the term-by-term chain rule (push),
    including strides that do not divide (the last rows/columns then receive no delta) and the
    negative numerators of the lower bound."""
    rng = np.random.default_rng(mi * 1000 + h * 100 + k * 10 + s)
    table = _rand_table(rng, mo, mi) if sparse else None
    n_conn = int(table.sum()) if sparse else mo * mi
    ho, wo = oracle.conv_out_size(h, k, s), oracle.conv_out_size(w, k, s)
    delta = rng.standard_normal((mo, ho, wo))
    wk = rng.standard_normal((n_conn, k, k))
    pull = ops.conv_backward(delta, wk, mi, h, w, k, k, s, s, table=table, push=False)
    push = ops.conv_backward(delta, wk, mi, h, w, k, k, s, s, table=table, push=True)
    np.testing.assert_allclose(pull, push, rtol=1e-12, atol=1e-12)
    # rows and columns that no kernel position reaches receive exactly zero
    reach_h = (ho - 1) * (s + 1) + k
    reach_w = (wo - 1) * (s + 1) + k
    assert (pull[:, reach_h:, :] == 0).all() and (pull[:, :, reach_w:] == 0).all()


@pytest.mark.parametrize("mi,mo,h,w,k,s,sparse", [(3, 4, 12, 11, 5, 1, False), (4, 5, 10, 10, 3, 0, True),
                                                  (2, 3, 13, 13, 4, 2, True), (3, 3, 9, 9, 2, 0, False)])
def test_conv_backward_and_weight_grad_vs_library_autograd(mi, mo, h, w, k, s, sparse):
    rng = np.random.default_rng(77 + k + s)
    table = _rand_table(rng, mo, mi) if sparse else np.ones((mo, mi), dtype=np.uint8)
    wk = rng.standard_normal((int(table.sum()), k, k))
    x = rng.standard_normal((mi, h, w))
    ho, wo = oracle.conv_out_size(h, k, s), oracle.conv_out_size(w, k, s)
    delta = rng.standard_normal((mo, ho, wo))
    xt = torch.from_numpy(x)[None].requires_grad_(True)
    wt = torch.from_numpy(_dense_from_csr(wk, table, k, k)).requires_grad_(True)
    bt = torch.zeros(mo, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.conv2d(xt, wt, bt, stride=s + 1).backward(torch.from_numpy(delta)[None])
    g_in = ops.conv_backward(delta, wk, mi, h, w, k, k, s, s, table=table if sparse else None)
    np.testing.assert_allclose(g_in, xt.grad[0].numpy(), rtol=1e-11, atol=1e-11)
    gb, gw = ops.conv_weight_grad(delta, x, k, k, s, s, table=table if sparse else None)
    np.testing.assert_allclose(gb, bt.grad.numpy(), rtol=1e-11, atol=1e-11)
    want = wt.grad.numpy()
    np.testing.assert_allclose(_dense_from_csr(gw, table, k, k), want * table[:, :, None, None],
                               rtol=1e-11, atol=1e-11)


def test_weight_grad_rectangular():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((2, 9, 11))
    delta = rng.standard_normal((3, oracle.conv_out_size(9, 2, 1), oracle.conv_out_size(11, 3, 0)))
    gb, gw = ops.conv_weight_grad(delta, x, 2, 3, 1, 0)
    xt = torch.from_numpy(x)[None]
    wt = torch.zeros(3, 2, 2, 3, dtype=torch.float64, requires_grad=True)
    torch.nn.functional.conv2d(xt, wt, stride=(2, 1)).backward(torch.from_numpy(delta)[None])
    np.testing.assert_allclose(gw.reshape(3, 2, 2, 3), wt.grad.numpy(), rtol=1e-11, atol=1e-11)


# ------------------------------------------------------------------ soft-max / cross-entropy

def test_softmax_xent_invariants():
    rng = np.random.default_rng(21)
    for n in (2, 5, 10):
        a = rng.standard_normal(n) * 3
        lab = int(rng.integers(n))
        e, p, d = ops.softmax_xent(a, lab)
        assert p.sum() == pytest.approx(1.0, rel=1e-14)
        assert d.sum() == pytest.approx(0.0, abs=1e-14)
        assert e >= 0 and e == pytest.approx(-np.log(p[lab]), rel=1e-14)
        # shift invariance, and the library's log-softmax
        e2, p2, _ = ops.softmax_xent(a + 100.0, lab)
        np.testing.assert_allclose(p2, p, rtol=1e-12)
        want = -torch.log_softmax(torch.from_numpy(a), 0)[lab].item()
        assert e == pytest.approx(want, rel=1e-12)
        # derivative by central differences
        for k in range(n):
            h = 1e-6
            ap, am = a.copy(), a.copy()
            ap[k] += h
            am[k] -= h
            fd = (ops.softmax_xent(ap, lab)[0] - ops.softmax_xent(am, lab)[0]) / (2 * h)
            assert d[k] == pytest.approx(fd, abs=1e-8)
    # uniform logits: p = 1/n, E = log n
    e, p, _ = ops.softmax_xent(np.zeros(4), 2)
    assert e == pytest.approx(np.log(4.0), rel=1e-14)
    # huge logits do not overflow
    e, p, _ = ops.softmax_xent(np.array([1000.0, 0.0]), 0)
    assert np.isfinite(e) and p[0] == pytest.approx(1.0)


# ------------------------------------------------------------------ scaled-tanh outputs / squared error

def test_tanh_sqerr_closed_forms_and_derivative():
    """The output variant with the paper's activation on the output neurons (Sec. 4) and the
    squared error against +-1 targets: values that follow from the definition alone."""
    A, B = 1.7159, 0.6666
    # zero pre-activations: y = 0, E = n/2, delta_k = -t_k * f'(0) = -t_k A B
    e, y, d = ops.tanh_sqerr(np.zeros(5), 3)
    assert e == pytest.approx(2.5, rel=1e-15)
    np.testing.assert_array_equal(y, np.zeros(5))
    want = np.full(5, A * B)
    want[3] = -A * B
    np.testing.assert_allclose(d, want, rtol=1e-14)
    # pre-activations that put every output on its target: E = 0, delta = 0
    a_one = np.arctanh(1.0 / A) / B
    a = np.full(4, -a_one)
    a[1] = a_one
    e, y, d = ops.tanh_sqerr(a, 1)
    assert e == pytest.approx(0.0, abs=1e-28)
    np.testing.assert_allclose(d, 0.0, atol=1e-14)
    # saturated and wrong: y -> -A on the class unit, error (A + 1)^2 / 2 from it alone, tiny delta
    e, y, d = ops.tanh_sqerr(np.array([-40.0, -a_one]), 0)
    assert e == pytest.approx((A + 1.0) ** 2 / 2, rel=1e-12)
    assert abs(d[0]) < 1e-12
    # general case: definition retyped with the library tanh, derivative by central differences
    rng = np.random.default_rng(33)
    for n in (2, 5, 10):
        a = rng.standard_normal(n) * 1.5
        lab = int(rng.integers(n))
        e, y, d = ops.tanh_sqerr(a, lab)
        t = -np.ones(n)
        t[lab] = 1.0
        yy = A * torch.tanh(B * torch.from_numpy(a)).numpy()
        np.testing.assert_allclose(y, yy, rtol=1e-14)
        assert e == pytest.approx(0.5 * np.sum((yy - t) ** 2), rel=1e-13)
        for k in range(n):
            h = 1e-6
            ap, am = a.copy(), a.copy()
            ap[k] += h
            am[k] -= h
            fd = (ops.tanh_sqerr(ap, lab)[0] - ops.tanh_sqerr(am, lab)[0]) / (2 * h)
            assert d[k] == pytest.approx(fd, abs=1e-8)
