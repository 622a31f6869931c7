"""Pins of the fp64 oracle against things other than itself (CPU only).

Each test names what it would catch.  References used: scalar-loop forward pass and
finite differences (tests/tiny_ref.py), torch float64 autograd on an independently
written model, hand-derived closed forms, numpy dense solves.
"""
import math

import numpy as np
import pytest
import torch

import dn_inputs
from oracle import dn_oracle as orc
from tests import tiny_ref

TINY_NETS = [
    (3, 2, 2),          # one hidden layer
    (4, 3, 3, 2),       # two hidden layers
    (2, 3, 2, 3, 2),    # three hidden layers
    (5, 3),             # no hidden layer
]


def _tiny(dims, l=6, s=4, C=0.7, seed=7):
    cfg = dn_inputs.custom(dims, l=l, s=s, C=C, seed=seed)
    X = dn_inputs.make_X(cfg).astype(np.float64)
    Y = dn_inputs.make_Y(cfg).astype(np.float64)
    theta = dn_inputs.make_theta(cfg, bias_scale=0.5).astype(np.float64)
    S = dn_inputs.make_subset(cfg)
    return cfg, X, Y, theta, S


def _torch_model(theta, dims):
    """Independent torch float64 model reading the theta layout of Section 2.1."""
    offs = dn_inputs.layer_offsets(dims)
    L = len(dims) - 1

    def f(th, X):
        z = X
        for m in range(1, L + 1):
            w, b = offs[m - 1]
            A = th[w:w + dims[m - 1] * dims[m]].reshape(dims[m], dims[m - 1])
            z = torch.nn.functional.linear(z, A, th[b:b + dims[m]])
            if m < L:
                z = torch.sigmoid(z)
        return z
    return f


# ------------------------------------------------------------------ forward / f

@pytest.mark.parametrize("dims", TINY_NETS)
def test_forward_and_f_match_scalar_loops(dims):
    # catches: transposed weight layout, bias offset errors, sigmoid on the output layer, 1/2 on the loss
    cfg, X, Y, theta, _ = _tiny(dims)
    Z = orc.forward(theta, dims, X)
    for i in range(X.shape[0]):
        np.testing.assert_allclose(Z[-1][i], tiny_ref.net_output(theta, dims, X[i]), rtol=1e-13, atol=1e-14)
    f = orc.loss(theta, dims, cfg.C, X, Y)
    assert abs(f - tiny_ref.objective(theta, dims, cfg.C, X, Y)) <= 1e-13 * abs(f)


def test_f_closed_form_one_weight():
    # 1-1 network, one sample: f = (w^2 + b^2)/(2C) + (w x + b - y)^2
    dims = (1, 1)
    w, b, x, y, C = 0.3, -0.2, 0.9, 1.0, 2.0
    f = orc.loss(np.array([w, b]), dims, C, np.array([[x]]), np.array([[y]]))
    assert abs(f - ((w * w + b * b) / (2 * C) + (w * x + b - y) ** 2)) < 1e-15


# ------------------------------------------------------------------ gradient

@pytest.mark.parametrize("dims", TINY_NETS)
def test_gradient_vs_finite_differences(dims):
    # catches: missing factor 2 in the seed, 1/l scaling, theta/C term, wrong sigma'
    cfg, X, Y, theta, _ = _tiny(dims)
    g, f = orc.grad(theta, dims, cfg.C, X, Y)
    g_fd = tiny_ref.fd_gradient(theta, dims, cfg.C, X, Y)
    assert np.linalg.norm(g - g_fd) <= 1e-7 * np.linalg.norm(g_fd)
    assert abs(f - tiny_ref.objective(theta, dims, cfg.C, X, Y)) <= 1e-13 * abs(f)


def test_gradient_vs_torch_autograd_config1():
    cfg = dn_inputs.config(1)
    X = dn_inputs.make_X(cfg).astype(np.float64)
    Y = dn_inputs.make_Y(cfg).astype(np.float64)
    theta = dn_inputs.make_theta(cfg, bias_scale=0.3).astype(np.float64)
    g, f = orc.grad(theta, cfg.dims, cfg.C, X, Y)
    th = torch.tensor(theta, requires_grad=True)
    model = _torch_model(theta, cfg.dims)
    ft = th @ th / (2 * cfg.C) + ((model(th, torch.tensor(X)) - torch.tensor(Y)) ** 2).sum() / cfg.l
    ft.backward()
    assert abs(f - ft.item()) <= 1e-13 * abs(f)
    np.testing.assert_allclose(g, th.grad.numpy(), rtol=1e-10, atol=1e-13)


# ------------------------------------------------------------------ Jacobian, J v, J^T w

@pytest.mark.parametrize("dims", TINY_NETS)
def test_jv_and_jt_vs_explicit_jacobian(dims):
    # catches: wrong Jacobian seed (identity, not the loss derivative), transposed operands in J^T
    cfg, X, Y, theta, S = _tiny(dims)
    XS = X[S]
    rng = np.random.default_rng(3)
    v = rng.standard_normal(theta.size)
    W = rng.standard_normal((XS.shape[0], dims[-1]))
    Z = orc.forward(theta, dims, XS)
    R = orc.jv(theta, dims, Z, v)
    acc = np.zeros(theta.size)
    for i in range(XS.shape[0]):
        J = tiny_ref.fd_jacobian(theta, dims, XS[i])
        np.testing.assert_allclose(R[i], J @ v, rtol=1e-7, atol=1e-9)
        acc += J.T @ W[i]
    got = orc._reverse_sweep(theta, dims, Z, W)
    assert np.linalg.norm(got - acc) <= 1e-7 * np.linalg.norm(acc)


def test_jacobian_vs_torch_autograd():
    dims = (4, 3, 3, 2)
    cfg, X, Y, theta, S = _tiny(dims)
    model = _torch_model(theta, dims)
    Z = orc.forward(theta, dims, X[S])
    for i in range(len(S)):
        xi = torch.tensor(X[S[i]])
        J = torch.autograd.functional.jacobian(lambda th: model(th, xi[None])[0], torch.tensor(theta)).numpy()
        for k in range(3):
            e = np.zeros(theta.size); e[5 * k + 1] = 1.0
            np.testing.assert_allclose(orc.jv(theta, dims, [z[i:i + 1] for z in Z], e)[0], J[:, 5 * k + 1],
                                       rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("dims", TINY_NETS)
def test_stored_blocks_are_output_derivatives_wrt_s(dims):
    # d z^L_u / d b^m_j = d z^L_u / d s^m_j (Section 3.3), so the bias columns of the
    # finite-difference Jacobian are the stored blocks; d z^L/d w^m_{tj} = P^m[u,j] z^{m-1}_t.
    cfg, X, Y, theta, S = _tiny(dims)
    XS = X[S]
    P = orc.jacobian_blocks(theta, dims, XS)
    Z = orc.forward(theta, dims, XS)
    offs = dn_inputs.layer_offsets(dims)
    L = len(dims) - 1
    for i in range(XS.shape[0]):
        J = tiny_ref.fd_jacobian(theta, dims, XS[i])
        for m in range(1, L + 1):
            w, b = offs[m - 1]
            np.testing.assert_allclose(P[m - 1][i], J[:, b:b + dims[m]], rtol=1e-7, atol=1e-9)
            Jw = J[:, w:w + dims[m - 1] * dims[m]].reshape(dims[-1], dims[m], dims[m - 1])
            np.testing.assert_allclose(Jw, P[m - 1][i][:, :, None] * Z[m - 1][i][None, None, :], rtol=1e-6, atol=1e-9)
    # closed forms: P^L = I, P^{L-1} = A^L diag(sigma'(s^{L-1}))
    np.testing.assert_array_equal(P[L - 1][0], np.eye(dims[-1]))
    if L >= 2:
        AL = orc.unpack(theta, dims)[L - 1][0]
        zi = Z[L - 1][1]
        np.testing.assert_allclose(P[L - 2][1], AL * (zi * (1 - zi))[None, :], rtol=1e-13)


def test_gradient_through_jacobian_identity():
    # Section 3.4: grad f = theta/C + (1/l) sum_i J_i^T 2 (z^{L,i} - y^i); on the subsample this
    # must equal back-propagation restricted to S.
    dims = (4, 3, 3, 2)
    cfg, X, Y, theta, S = _tiny(dims)
    XS, YS = X[S], Y[S]
    g, _ = orc.grad(theta, dims, cfg.C, XS, YS)
    acc = theta / cfg.C
    for i in range(len(S)):
        J = tiny_ref.fd_jacobian(theta, dims, XS[i])
        z = np.array(tiny_ref.net_output(theta, dims, XS[i]))
        acc = acc + J.T @ (2.0 * (z - YS[i])) / len(S)
    assert np.linalg.norm(g - acc) <= 1e-7 * np.linalg.norm(acc)


# ------------------------------------------------------------------ Gauss-Newton products

@pytest.mark.parametrize("dims", TINY_NETS)
def test_gn_matvec_vs_dense_brute_force(dims):
    # catches: B = I instead of 2I, 1/l instead of 1/|S|, missing v/C
    cfg, X, Y, theta, S = _tiny(dims)
    XS = X[S]
    G = tiny_ref.dense_gauss_newton(theta, dims, cfg.C, XS)
    rng = np.random.default_rng(5)
    for _ in range(3):
        v = rng.standard_normal(theta.size)
        got = orc.gn_matvec(theta, dims, cfg.C, XS, v)
        assert np.linalg.norm(got - G @ v) <= 1e-7 * np.linalg.norm(G @ v)


@pytest.mark.parametrize("dims", TINY_NETS)
def test_blockdiag_matvec_vs_dense_block_diagonal(dims):
    cfg, X, Y, theta, S = _tiny(dims)
    XS = X[S]
    G = tiny_ref.dense_gauss_newton(theta, dims, cfg.C, XS)
    Ghat = tiny_ref.zero_offdiag_layer_blocks(G, dims)
    v = np.random.default_rng(6).standard_normal(theta.size)
    got = orc.gn_matvec_blockdiag(theta, dims, cfg.C, XS, v)
    assert np.linalg.norm(got - Ghat @ v) <= 1e-7 * np.linalg.norm(Ghat @ v)
    if len(dims) > 2:
        assert np.linalg.norm(Ghat @ v - G @ v) > 1e-3 * np.linalg.norm(G @ v)  # the two operators differ


def test_blockdiag_equals_full_on_single_block_support_and_for_L1():
    dims = (4, 3, 3, 2)
    cfg, X, Y, theta, S = _tiny(dims)
    XS = X[S]
    rng = np.random.default_rng(8)
    for sl in orc.block_slices(dims):
        v = np.zeros(theta.size)
        v[sl] = rng.standard_normal(sl.stop - sl.start)
        full = orc.gn_matvec(theta, dims, cfg.C, XS, v)
        hat = orc.gn_matvec_blockdiag(theta, dims, cfg.C, XS, v)
        np.testing.assert_allclose(hat[sl], full[sl], rtol=1e-12, atol=1e-14)
    dims1 = (5, 3)
    cfg, X, Y, theta, S = _tiny(dims1)
    v = rng.standard_normal(theta.size)
    np.testing.assert_allclose(orc.gn_matvec_blockdiag(theta, dims1, cfg.C, X[S], v),
                               orc.gn_matvec(theta, dims1, cfg.C, X[S], v), rtol=1e-13)


def test_gn_symmetry_and_definiteness_config1():
    cfg = dn_inputs.config(1)
    X = dn_inputs.make_X(cfg).astype(np.float64)
    theta = dn_inputs.make_theta(cfg, bias_scale=0.3).astype(np.float64)
    XS = X[dn_inputs.make_subset(cfg)]
    v = dn_inputs.make_probe(cfg, 0).astype(np.float64)
    w = dn_inputs.make_probe(cfg, 1).astype(np.float64)
    for product in (orc.gn_matvec, orc.gn_matvec_blockdiag):
        Gv = product(theta, cfg.dims, cfg.C, XS, v)
        Gw = product(theta, cfg.dims, cfg.C, XS, w)
        assert abs(w @ Gv - v @ Gw) <= 1e-12 * abs(w @ Gv)
        assert v @ Gv >= v @ v / cfg.C
    # v^T G v = v^T v / C + (2/|S|) sum_i ||J_i v||^2
    Z = orc.forward(theta, cfg.dims, XS)
    R = orc.jv(theta, cfg.dims, Z, v)
    Gv = orc.gn_matvec(theta, cfg.dims, cfg.C, XS, v)
    assert abs(v @ Gv - (v @ v / cfg.C + 2.0 * np.sum(R * R) / XS.shape[0])) <= 1e-12 * abs(v @ Gv)


def test_gn_closed_form_scalar_network():
    # 1-1-1 network, one sample: J = [w2 s' x, w2 s', z1, 1] with z1 = sigmoid(w1 x + b1), s' = z1(1-z1);
    # G = I/C + 2 J^T J.
    dims = (1, 1, 1)
    w1, b1, w2, b2, x, C = 0.4, -0.1, 0.8, 0.2, 0.6, 3.0
    z1 = 1.0 / (1.0 + math.exp(-(w1 * x + b1)))
    sp = z1 * (1 - z1)
    J = np.array([w2 * sp * x, w2 * sp, z1, 1.0])
    G = np.eye(4) / C + 2.0 * np.outer(J, J)
    v = np.array([1.0, -2.0, 0.5, 3.0])
    got = orc.gn_matvec(np.array([w1, b1, w2, b2]), dims, C, np.array([[x]]), v)
    np.testing.assert_allclose(got, G @ v, rtol=1e-13)


# ------------------------------------------------------------------ no hidden layer: ridge regression

def test_no_hidden_layer_newton_step_is_ridge_solution():
    # z = A x + b is linear in theta, so G is the exact Hessian and one undamped Newton step with
    # S = all samples lands on the minimiser of f, which for each output u solves
    # (I/C + (2/l) Xt^T Xt) [a_u; b_u] = (2/l) Xt^T y_u with Xt = [X, 1].
    dims = (5, 3)
    cfg, X, Y, theta, _ = _tiny(dims, l=12, s=12, C=2.5)
    l = X.shape[0]
    Xt = np.hstack([X, np.ones((l, 1))])
    H = np.eye(6) / cfg.C + 2.0 / l * Xt.T @ Xt
    sol = np.linalg.solve(H, 2.0 / l * Xt.T @ Y)           # [6, 3]: column u = [a_u; b_u]
    theta_star = np.concatenate([sol[:5, :].T.ravel(), sol[5, :]])
    g, _ = orc.grad(theta, dims, cfg.C, X, Y)
    d, iters, res = orc.cg(theta, dims, cfg.C, X, g, lam=0.0, max_iter=theta.size + 2, sigma=1e-13)
    np.testing.assert_allclose(theta + d, theta_star, rtol=1e-9, atol=1e-11)
    g_star, _ = orc.grad(theta_star, dims, cfg.C, X, Y)
    assert np.linalg.norm(g_star) <= 1e-12 * max(1.0, np.linalg.norm(g))


# ------------------------------------------------------------------ CG

@pytest.mark.parametrize("blockdiag", [False, True])
def test_cg_converges_to_dense_solve(blockdiag):
    dims = (4, 3, 3, 2)
    cfg, X, Y, theta, S = _tiny(dims)
    XS = X[S]
    lam = 0.3
    g, _ = orc.grad(theta, dims, cfg.C, X, Y)
    G = tiny_ref.dense_gauss_newton(theta, dims, cfg.C, XS)
    if blockdiag:
        G = tiny_ref.zero_offdiag_layer_blocks(G, dims)
    d_ref = np.linalg.solve(G + lam * np.eye(theta.size), -g)
    d, iters, res = orc.cg(theta, dims, cfg.C, XS, g, lam, max_iter=4 * theta.size, sigma=1e-12, blockdiag=blockdiag)
    assert np.linalg.norm(d - d_ref) <= 1e-6 * np.linalg.norm(d_ref)
    # recurrence residual agrees with the recomputed one
    prod = orc.gn_matvec_blockdiag if blockdiag else orc.gn_matvec
    true_res = prod(theta, dims, cfg.C, XS, d) + lam * d + g
    blocks = orc.block_slices(dims) if blockdiag else [slice(0, theta.size)]
    assert len(res) == len(blocks)
    for k, b in enumerate(blocks):
        assert abs(np.linalg.norm(true_res[b]) - res[k]) <= 1e-6 * np.linalg.norm(g[b])
        assert res[k] <= 1e-12 * np.linalg.norm(g[b]) * 1.0001


def test_cg_first_step_closed_form_and_fixed_iteration_count():
    cfg = dn_inputs.config(1)
    X = dn_inputs.make_X(cfg).astype(np.float64)
    Y = dn_inputs.make_Y(cfg).astype(np.float64)
    theta = dn_inputs.make_theta(cfg, bias_scale=0.3).astype(np.float64)
    XS = X[dn_inputs.make_subset(cfg)]
    g, _ = orc.grad(theta, cfg.dims, cfg.C, X, Y)
    Ag = orc.gn_matvec(theta, cfg.dims, cfg.C, XS, g) + cfg.lam * g
    d1, it, _ = orc.cg(theta, cfg.dims, cfg.C, XS, g, cfg.lam, max_iter=1)
    assert it == 1
    np.testing.assert_allclose(d1, -(g @ g) / (g @ Ag) * g, rtol=1e-12)
    # sigma = 0 never stops early; iterates decrease the quadratic model monotonically
    d, it, res, hist = orc.cg(theta, cfg.dims, cfg.C, XS, g, cfg.lam, max_iter=cfg.cg_iters, history=True)
    assert it == cfg.cg_iters and len(hist) == cfg.cg_iters

    def model(dd):
        return 0.5 * dd @ (orc.gn_matvec(theta, cfg.dims, cfg.C, XS, dd) + cfg.lam * dd) + g @ dd
    vals = [model(h) for h in hist]
    assert all(b < a for a, b in zip(vals, vals[1:]))


def test_cg_blockdiag_blocks_stop_independently():
    dims = (4, 3, 3, 2)
    cfg, X, Y, theta, S = _tiny(dims)
    g, _ = orc.grad(theta, dims, cfg.C, X, Y)
    d, iters, res = orc.cg(theta, dims, cfg.C, X[S], g, 0.5, max_iter=200, sigma=1e-3, blockdiag=True)
    for k, b in enumerate(orc.block_slices(dims)):
        assert res[k] <= 1e-3 * np.linalg.norm(g[b])
    # each block equals CG run on that block alone
    for k, b in enumerate(orc.block_slices(dims)):
        gk = np.zeros_like(g); gk[b] = g[b]
        dk, _, _ = orc.cg(theta, dims, cfg.C, X[S], gk, 0.5, max_iter=200, sigma=1e-3, blockdiag=True)
        np.testing.assert_allclose(d[b], dk[b], rtol=1e-12, atol=1e-15)


def test_variable_partitions_follow_the_papers_example():
    # Section 3.1: a 150-200-30 network split 3-2-3 has 12 partitions; (A0, A1) holds a 50 x 100 block of W^1;
    # the 200 biases of layer 1 are split 100 / 100 between the two partitions of the FIRST input group
    dims, split = (150, 200, 30), (3, 2, 3)
    sets = orc.partition_index_sets(dims, split)
    assert len(sets) == 12
    n = orc.num_params(dims)
    allidx = np.concatenate(sets)
    assert allidx.size == n and np.array_equal(np.sort(allidx), np.arange(n))      # a partition of the variables
    sizes = [s.size for s in sets]
    assert sizes[:6] == [50 * 100 + 100, 50 * 100 + 100, 50 * 100, 50 * 100, 50 * 100, 50 * 100]
    assert sizes[6:] == [100 * 10 + 10] * 3 + [100 * 10] * 3
    # element check with the index formula of Section 2.1: w^1_{tj} at j * 150 + t
    A01 = set(sets[1].tolist())                     # (a = 0, b = 1): t in 0..49, j in 100..199
    assert (100 * 150 + 0) in A01 and (199 * 150 + 49) in A01 and (100 * 150 + 50) not in A01
    assert (150 * 200 + 100) in A01 and (150 * 200 + 99) not in A01              # bias b^1_100
    # one group everywhere = one partition per layer
    for sl, idx in zip(orc.block_slices(dims), orc.partition_index_sets(dims, (1, 1, 1))):
        assert np.array_equal(np.sort(idx), np.arange(sl.start, sl.stop))


@pytest.mark.parametrize("dims,split", [((4, 3, 3, 2), (2, 1, 3, 1)), ((5, 4, 3), (3, 2, 2)), ((6, 4), (2, 3))])
def test_partitioned_product_is_the_block_diagonal_of_dense_G(dims, split):
    # catches: biases assigned to the wrong partition, cross-partition terms kept, wrong group boundaries
    cfg, X, Y, theta, S = _tiny(dims, l=8, s=5)
    XS = X[S]
    G = tiny_ref.dense_gauss_newton(theta, dims, cfg.C, XS)
    # membership map built here from the paper's description, not from the oracle's index sets
    owner = np.empty(G.shape[0], dtype=np.int64)
    o, pid = 0, 0
    for m in range(1, len(dims)):
        nprev, ncur = dims[m - 1], dims[m]
        ga = [(k * nprev) // split[m - 1] for k in range(split[m - 1] + 1)]
        gb = [(k * ncur) // split[m] for k in range(split[m] + 1)]
        grp_prev = np.searchsorted(ga, np.arange(nprev), side="right") - 1
        grp_cur = np.searchsorted(gb, np.arange(ncur), side="right") - 1
        for j in range(ncur):
            for t in range(nprev):
                owner[o + j * nprev + t] = pid + grp_prev[t] * split[m] + grp_cur[j]
            owner[o + nprev * ncur + j] = pid + 0 * split[m] + grp_cur[j]
        o += nprev * ncur + ncur
        pid += split[m - 1] * split[m]
    Ghat = np.where(owner[:, None] == owner[None, :], G, 0.0)
    rng = np.random.default_rng(3)
    for _ in range(3):
        v = rng.standard_normal(G.shape[0])
        np.testing.assert_allclose(orc.gn_matvec_partitioned(theta, dims, cfg.C, XS, v, split), Ghat @ v,
                                   rtol=2e-6, atol=1e-8)
    # CG over the partitions solves the block-diagonal system
    g, _ = orc.grad(theta, dims, cfg.C, X, Y)
    d, it, res = orc.cg(theta, dims, cfg.C, XS, g, 0.2, 300, sigma=1e-12, blockdiag=True, split=split)
    np.testing.assert_allclose(d, np.linalg.solve(Ghat + 0.2 * np.eye(G.shape[0]), -g), rtol=1e-6, atol=1e-9)
    assert len(res) == sum(split[m - 1] * split[m] for m in range(1, len(dims)))
    # with one group per layer it is the per-layer product
    v = rng.standard_normal(G.shape[0])
    np.testing.assert_allclose(orc.gn_matvec_partitioned(theta, dims, cfg.C, XS, v, (1,) * len(dims)),
                               orc.gn_matvec_blockdiag(theta, dims, cfg.C, XS, v), rtol=1e-13, atol=1e-15)


def test_cg_early_termination_across_blocks():
    # catches: the percentage applied to running instead of finished blocks, cg_min ignored, a finished block
    # still being updated, the rule leaking into the single-system mode
    dims = (12, 10, 8, 3)
    cfg, X, Y, theta, S = _tiny(dims, l=80, s=60, C=100.0, seed=23)
    XS = X[S]
    g, _ = orc.grad(theta, dims, cfg.C, X, Y)
    blocks = orc.block_slices(dims)
    lam, sigma = 1e-3, 1e-6
    # iteration at which each block meets its own test when run alone (independent of the rule under test)
    own = []
    for b in blocks:
        gk = np.zeros_like(g); gk[b] = g[b]
        _, it, _, hist = orc.cg(theta, dims, cfg.C, XS, gk, lam, 500, sigma=sigma, blockdiag=True, history=True)
        own.append(it)
    own_sorted = sorted(own)
    assert len(set(own)) == 3                  # the three blocks finish at different iterations
    _, it_all, _ = orc.cg(theta, dims, cfg.C, XS, g, lam, 500, sigma=sigma, blockdiag=True)
    assert it_all == own_sorted[-1]
    for r, expect in ((100.0, own_sorted[2]), (67.0, own_sorted[2]), (66.0, own_sorted[1]), (34.0, own_sorted[1]),
                      (33.0, own_sorted[0]), (1.0, own_sorted[0])):
        d, it, res = orc.cg(theta, dims, cfg.C, XS, g, lam, 500, sigma=sigma, blockdiag=True, cg_min=0, r_percent=r)
        assert it == expect, (r, it, expect)
    # cg_min delays the joint stop but not a block's own stop
    cg_min = own_sorted[0] + 1
    assert cg_min < own_sorted[1]
    d, it, res, hist = orc.cg(theta, dims, cfg.C, XS, g, lam, 500, sigma=sigma, blockdiag=True, cg_min=cg_min,
                              r_percent=1.0, history=True)
    assert it == cg_min
    first = own.index(own_sorted[0])
    np.testing.assert_array_equal(hist[-1][blocks[first]], hist[own_sorted[0] - 1][blocks[first]])   # frozen since
    # blocks cut short equal their own iterates at that count
    for k, b in enumerate(blocks):
        gk = np.zeros_like(g); gk[b] = g[b]
        dk, _, _ = orc.cg(theta, dims, cfg.C, XS, gk, lam, min(cg_min, own[k]), sigma=0.0, blockdiag=True)
        np.testing.assert_allclose(d[b], dk[b], rtol=1e-12, atol=1e-15)
    # the single-system mode ignores the rule
    d1, it1, _ = orc.cg(theta, dims, cfg.C, XS, g, lam, 50, sigma=0.0, blockdiag=False, r_percent=1.0)
    assert it1 == 50


# ------------------------------------------------------------------ outer Newton iteration

def test_direction_combination_minimises_the_two_variable_model():
    # catches: lambda leaking into the matrix, swapped right-hand sides, the block-diagonal matrix used
    # instead of the whole one, wrong sign of the right-hand side
    dims = (4, 3, 3, 2)
    cfg, X, Y, theta, S = _tiny(dims, l=12, s=8)
    XS = X[S]
    g, _ = orc.grad(theta, dims, cfg.C, X, Y)
    rng = np.random.default_rng(5)
    d = -g + 0.1 * rng.standard_normal(g.size)
    d_bar = rng.standard_normal(g.size)
    b1, b2, (a11, a12, a22) = orc.combine_directions(theta, dims, cfg.C, XS, g, d, d_bar, eps=1e-12)
    G = tiny_ref.dense_gauss_newton(theta, dims, cfg.C, XS)
    np.testing.assert_allclose([a11, a12, a22], [d @ G @ d, d_bar @ G @ d, d_bar @ G @ d_bar], rtol=1e-6)

    def model(x, y):
        u = x * d + y * d_bar
        return 0.5 * u @ G @ u + g @ u
    best = model(b1, b2)
    for dx in (-1e-2, 0.0, 1e-2):
        for dy in (-1e-2, 0.0, 1e-2):
            assert model(b1 + dx, b2 + dy) >= best - 1e-12
    # least squares over the span of {d, d_bar} gives the same coefficients
    D = np.stack([d, d_bar], axis=1)
    coef = np.linalg.solve(D.T @ G @ D, -D.T @ g)
    np.testing.assert_allclose([b1, b2], coef, rtol=1e-5)
    # a zero previous direction (first iteration) or a parallel one is ill-conditioned: keep d
    assert orc.combine_directions(theta, dims, cfg.C, XS, g, d, np.zeros_like(d))[:2] == (1.0, 0.0)
    assert orc.combine_directions(theta, dims, cfg.C, XS, g, d, 2.0 * d, eps=1e-9)[:2] == (1.0, 0.0)


def test_line_search_returns_the_largest_admissible_power_of_one_half():
    # catches: accepting the first alpha, a missing eta term, halving before the first trial
    dims = (4, 3, 3, 2)
    cfg, X, Y, theta, S = _tiny(dims, l=12, s=8)
    g, f0 = orc.grad(theta, dims, cfg.C, X, Y)
    eta = 1e-2
    for scale in (0.5, 20.0, 150.0):             # the largest scales overshoot and force several halvings
        d = -scale * g
        gTd = float(g @ d)
        alpha, f_new, evals = orc.line_search(theta, dims, cfg.C, X, Y, f0, gTd, d, eta=eta)
        ok = [tiny_ref.objective(theta + 0.5 ** k * d, dims, cfg.C, X, Y) <= f0 + eta * 0.5 ** k * gTd
              for k in range(30)]
        first = ok.index(True)
        assert alpha == 0.5 ** first and evals == first + 1
        assert abs(f_new - tiny_ref.objective(theta + alpha * d, dims, cfg.C, X, Y)) <= 1e-12 * abs(f_new)
    assert first >= 2                            # the scan really had rejections to get past
    # an ascent direction is never accepted
    alpha, f_new, evals = orc.line_search(theta, dims, cfg.C, X, Y, f0, float(g @ g), g, eta=eta, max_trials=8)
    assert alpha == 0.0 and f_new == f0 and evals == 8


def test_levenberg_marquardt_rule_table():
    assert orc.lm_update(3.0, 0.76, drop=0.5, boost=4.0) == 1.5
    assert orc.lm_update(3.0, 0.75, drop=0.5, boost=4.0) == 3.0
    assert orc.lm_update(3.0, 0.25, drop=0.5, boost=4.0) == 3.0
    assert orc.lm_update(3.0, 0.2499, drop=0.5, boost=4.0) == 12.0
    assert orc.lm_update(3.0, -2.0, drop=0.5, boost=4.0) == 12.0
    assert orc.lm_update(1.0, 0.9) == pytest.approx(2.0 / 3.0) and orc.lm_update(1.0, 0.1) == 1.5


def test_newton_step_is_exact_on_the_ridge_problem():
    # no hidden layer: f is quadratic and G is its Hessian, so one undamped step over all samples lands on
    # the minimiser, the full step is accepted, and actual reduction = predicted reduction (rho = 1)
    dims = (5, 3)
    cfg, X, Y, theta, _ = _tiny(dims, l=40, s=40, C=2.0)
    S = np.arange(40)
    n = theta.size
    out = orc.newton_step(theta, dims, cfg.C, X, Y, S, np.zeros(n), lam=0.0, cg_max=200, sigma=1e-14,
                          eta=1e-4, drop=0.5, boost=4.0)
    Xa = np.hstack([X, np.ones((40, 1))])
    Wopt = np.linalg.solve(np.eye(6) / cfg.C + 2.0 / 40 * Xa.T @ Xa, 2.0 / 40 * Xa.T @ Y)     # [6 x 3]
    theta_opt = np.concatenate([Wopt[:5].T.ravel(), Wopt[5]])
    np.testing.assert_allclose(out["theta"], theta_opt, rtol=1e-8, atol=1e-10)
    assert out["alpha"] == 1.0 and out["f_evals"] == 1 and out["beta"] == (1.0, 0.0)
    assert abs(out["rho"] - 1.0) <= 1e-9
    assert out["lam"] == 0.0
    assert abs(out["f_new"] - tiny_ref.objective(theta_opt, dims, cfg.C, X, Y)) <= 1e-12
    # predicted reduction pieces: g'd = -d'Gd at the exact Newton direction
    assert abs(out["gTd"] + out["dGd"]) <= 1e-9 * abs(out["dGd"])


@pytest.mark.parametrize("blockdiag", [False, True])
def test_newton_iterations_decrease_f_and_follow_the_rules(blockdiag):
    # catches: theta not advanced, d_prev not carried, lambda updated from the wrong ratio
    dims = (6, 5, 4, 3)
    cfg, X, Y, theta, _ = _tiny(dims, l=60, s=20, C=5.0, seed=11)
    d_prev = np.zeros(theta.size)
    lam = 1.0
    fs = [orc.loss(theta, dims, cfg.C, X, Y)]
    used_prev = False
    for k in range(4):
        S = np.random.default_rng(100 + k).permutation(60)[:20]
        out = orc.newton_step(theta, dims, cfg.C, X, Y, S, d_prev, lam, cg_max=30, sigma=1e-3, blockdiag=blockdiag)
        assert abs(out["f_old"] - fs[-1]) <= 1e-13 * abs(fs[-1])
        assert out["alpha"] > 0 and out["f_new"] <= out["f_old"] + 1e-4 * out["alpha"] * out["gTd"]
        assert out["gTd"] < 0
        np.testing.assert_allclose(out["theta"], theta + out["alpha"] * out["d"], rtol=1e-14, atol=1e-16)
        rho = (out["f_new"] - out["f_old"]) / (out["alpha"] * out["gTd"] + 0.5 * out["alpha"] ** 2 * out["dGd"])
        assert abs(rho - out["rho"]) <= 1e-12 * abs(rho)
        assert out["lam"] == orc.lm_update(lam, rho)
        # d'Gd reported for the combined direction is the quadratic form of the whole matrix
        Gd = orc.gn_matvec(theta, dims, cfg.C, X[S], out["d"])
        assert abs(out["d"] @ Gd - out["dGd"]) <= 1e-9 * abs(out["dGd"])
        if k == 0:
            assert out["beta"] == (1.0, 0.0)
        used_prev |= out["beta"][1] != 0.0
        theta, d_prev, lam = out["theta"], out["d"], out["lam"]
        fs.append(out["f_new"])
    assert all(b < a for a, b in zip(fs, fs[1:]))
    assert used_prev


# ------------------------------------------------------------------ inputs

def test_input_generator_shapes_and_ranges():
    cfg = dn_inputs.config(1)
    X = dn_inputs.make_X(cfg)
    assert X.dtype == np.float32 and X.shape == (200, 20) and X.min() >= 0.0 and X.max() < 1.0
    Y = dn_inputs.make_Y(cfg)
    assert Y.shape == (200, 4) and np.all(Y.sum(axis=1) == 1.0)
    S = dn_inputs.make_subset(cfg)
    assert S.shape == (50,) and len(set(S.tolist())) == 50 and S.min() >= 0 and S.max() < 200
    th = dn_inputs.make_theta(cfg)
    assert th.shape == (676,) and cfg.n_params == 676
    a = math.sqrt(6.0 / 36)
    assert np.abs(th[:320]).max() <= a and np.all(th[320:336] == 0)
    np.testing.assert_array_equal(dn_inputs.make_X(cfg, rows=10), X[:10])
    c4 = dn_inputs.custom((6, 4), l=1000, s=10, features="normal3")
    X4 = dn_inputs.make_X(c4)
    assert X4.min() >= -3.0 and X4.max() <= 3.0 and abs(float(X4.mean())) < 0.1
    assert [dn_inputs.config(i).n_params for i in range(1, 6)] == [676, 328810, 3578510, 12302100, 71222248]
    # sparse initialisation: ceil(sqrt(n_{m-1})) non-zero weights into every neuron, zero biases
    cs = dn_inputs.custom((50, 17, 10, 3), l=10, s=5)
    ths = dn_inputs.make_theta(cs, init="sparse")
    for m, (w, b) in enumerate(dn_inputs.layer_offsets(cs.dims), start=1):
        A = ths[w:w + cs.dims[m - 1] * cs.dims[m]].reshape(cs.dims[m], cs.dims[m - 1])
        assert np.all((A != 0).sum(axis=1) == math.ceil(math.sqrt(cs.dims[m - 1])))
        assert np.all(ths[b:b + cs.dims[m]] == 0)
    assert [math.ceil(math.sqrt(k)) for k in (50, 17, 10)] == [8, 5, 4]
    # dense initialisation: per-layer standard deviations 0.1 / 0.05 / 0.001
    cd = dn_inputs.custom((400, 300, 200, 100), l=10, s=5)
    thd = dn_inputs.make_theta(cd, init="dense")
    sds = [thd[w:w + cd.dims[m] * cd.dims[m + 1]].std() for m, (w, _) in enumerate(dn_inputs.layer_offsets(cd.dims))]
    np.testing.assert_allclose(sds, [0.1, 0.05, 0.001], rtol=0.02)


def test_partition_counts_match_the_papers_table():
    """Every (network, split structure) pair the paper prints gives the printed number of partitions, the
    partitions tile the variables exactly once, each holds |T_{m-1}| x |T_m| weights (plus the biases of its
    output group when it belongs to the first input group), and the Pendigits weight counts come out as printed."""
    from tests.golden_io import split_structures
    rows, weights = split_structures()
    assert len(rows) == 10
    by_name = {}
    for name, dims, split, count in rows:
        sets = orc.partition_index_sets(dims, split)
        assert len(sets) == count, name
        n = orc.num_params(dims)
        seen = np.zeros(n, dtype=np.int8)
        for idx in sets:
            seen[idx] += 1
        assert np.all(seen == 1), name
        w_counts, k = [], 0
        for m in range(1, len(dims)):
            ba, bb = orc.group_bounds(dims[m - 1], split[m - 1]), orc.group_bounds(dims[m], split[m])
            for a in range(split[m - 1]):
                for b in range(split[m]):
                    w = (ba[a + 1] - ba[a]) * (bb[b + 1] - bb[b])
                    assert sets[k].size == w + ((bb[b + 1] - bb[b]) if a == 0 else 0), (name, m, a, b)
                    w_counts.append(w)
                    k += 1
        by_name[name] = w_counts
    for name, largest, smallest in weights:
        assert max(by_name[name]) == largest and min(by_name[name]) == smallest
